// fp32 GEMM for the fp32 reference-precision path (tiny shapes, any sizes):
// LDS-tiled FMA kernel, 64x64 output tile, fully guarded edges, fp32 throughout.
#include "common.h"
#include "kernels.h"

namespace hh {

constexpr int FT = 64;   // tile edge
constexpr int FK = 16;   // k step

// A(m,k) = A[m*sam + k*sak], B(n,k) = B[n*sbn + k*sbk]; AK/BK: k is the contiguous index.
template <bool AK, bool BK>
__global__ __launch_bounds__(256) void k_gemm_f32(const float* __restrict__ A, long sam, long sak,
                                                  const float* __restrict__ B, long sbn, long sbk,
                                                  float* __restrict__ C, int ldc, const float* __restrict__ R, int ldr,
                                                  int M, int N, int K, int accumulate) {
    __shared__ float As[FK][FT + 4];
    __shared__ float Bs[FK][FT + 4];
    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    const int m0 = blockIdx.y * FT, n0 = blockIdx.x * FT;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += FK) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int idx = tid + 256 * i;
            {
                const int mm = AK ? idx / FK : idx % FT, kk = AK ? idx % FK : idx / FT;
                const int gm = m0 + mm, gk = k0 + kk;
                As[kk][mm] = (gm < M && gk < K) ? A[gm * sam + gk * sak] : 0.f;
            }
            {
                const int nn = BK ? idx / FK : idx % FT, kk = BK ? idx % FK : idx / FT;
                const int gn = n0 + nn, gk = k0 + kk;
                Bs[kk][nn] = (gn < N && gk < K) ? B[gn * sbn + gk * sbk] : 0.f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < FK; kk++) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; i++) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int gn = n0 + tx * 4 + j;
            if (gn >= N) continue;
            float v = acc[i][j];
            if (R) v += R[(size_t)gm * ldr + gn];
            float* c = C + (size_t)gm * ldc + gn;
            *c = accumulate ? *c + v : v;
        }
    }
}

hipError_t gemm_f32(const GemmDesc& g, hipStream_t st) {
    dim3 grid((g.N + FT - 1) / FT, (g.M + FT - 1) / FT);
    const float* A = (const float*)g.A;
    const float* B = (const float*)g.B;
    float* C = (float*)g.C;
    const float* R = (const float*)g.R;
    switch (g.kind) {
        case GEMM_NT:
            k_gemm_f32<true, true><<<grid, 256, 0, st>>>(A, g.lda, 1, B, g.ldb, 1, C, g.ldc, R, g.ldr, g.M, g.N, g.K, g.accumulate);
            break;
        case GEMM_NN:
            k_gemm_f32<true, false><<<grid, 256, 0, st>>>(A, g.lda, 1, B, 1, g.ldb, C, g.ldc, R, g.ldr, g.M, g.N, g.K, g.accumulate);
            break;
        case GEMM_TN:
            k_gemm_f32<false, false><<<grid, 256, 0, st>>>(A, 1, g.lda, B, 1, g.ldb, C, g.ldc, R, g.ldr, g.M, g.N, g.K, g.accumulate);
            break;
        default:
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace hh
