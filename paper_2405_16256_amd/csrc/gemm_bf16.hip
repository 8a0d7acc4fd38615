// bf16 x bf16 -> fp32 GEMMs on the gfx950 matrix cores for the projections of the
// decoder layer and their input / weight gradients.
//
//   NT  C[M,N] = A[M,K] B[N,K]^T      forward  y  = x W^T
//   NN  C[M,N] = A[M,K] B[K,N]        backward dX = dY W
//   TN  C[M,N] = A[K,M]^T B[K,N]      backward dW = dY^T X   (fp32 output, optional +=)
//
// One workgroup = 4 waves in a 2x2 grid computes a BM x BN tile of C with
// v_mfma_f32_32x32x16_bf16; the k loop advances 64 at a time through two LDS
// stages, the next tile's global loads (buffer loads: rows past the end of a
// tensor read as zero) in flight while the current one feeds the matrix cores.
//
// Operand tiles in LDS keep the layout they have in memory, so every global
// load and LDS store is a 16-byte access:
//   * k contiguous in memory  -> LDS [row][64 k], 16-byte chunks XOR-swizzled by
//     the row index; fragments come out with ds_read_b128.
//   * k strided in memory     -> LDS [64 k][rows], 64-byte slots XOR-swizzled by
//     the k index; fragments come out with the transposing ds_read_b64_tr_b16.
// Either way lane l of a fragment holds row (l % 32), k = 16*step + 8*(l/32) .. +7.
//
// The MFMA takes the B-side fragment as its first operand, so each accumulator
// lane owns one row m of C and runs of 4 consecutive columns n: stores are 8-byte
// (bf16) or 16-byte (fp32) vectors along the contiguous dimension of C.
#include "common.h"
#include "kernels.h"

namespace hh {

constexpr int GK = 64;        // k tile
constexpr int GTHREADS = 256;

template <int ROWS, bool KC>
struct TileLoader {
    static constexpr int CHUNKS = ROWS * GK / 8;          // 16-byte chunks per tile
    static constexpr int PER_THREAD = CHUNKS / GTHREADS;
    static_assert(CHUNKS % GTHREADS == 0, "tile must split evenly over the workgroup");

    // global byte offset of chunk c of the tile at (row0, k0)
    __device__ static __forceinline__ uint32_t goff(int c, int row0, int k0, int ld) {
        if (KC) {
            const int r = c >> 3, ch = c & 7;
            return ((uint32_t)(row0 + r) * (uint32_t)ld + (uint32_t)(k0 + ch * 8)) * 2u;
        } else {
            constexpr int CPR = ROWS / 8;
            const int k = c / CPR, rc = c % CPR;
            return ((uint32_t)(k0 + k) * (uint32_t)ld + (uint32_t)(row0 + rc * 8)) * 2u;
        }
    }
    // LDS byte offset of chunk c
    __device__ static __forceinline__ int loff(int c) {
        if (KC) {
            const int r = c >> 3, ch = c & 7;
            return r * 128 + ((ch ^ ((r >> 1) & 7)) << 4);
        } else {
            constexpr int CPR = ROWS / 8;
            const int k = c / CPR, rc = c % CPR;
            return k * (ROWS * 2) + ((rc * 16) ^ ((k & 3) << 6));
        }
    }
    __device__ static __forceinline__ void load(i32x4 (&st)[PER_THREAD], __amdgpu_buffer_rsrc_t rs, int row0, int k0, int ld) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; i++)
            st[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, goff(threadIdx.x + GTHREADS * i, row0, k0, ld), 0, 0);
    }
    __device__ static __forceinline__ void store(const i32x4 (&st)[PER_THREAD], char* lds) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; i++)
            *reinterpret_cast<i32x4*>(lds + loff(threadIdx.x + GTHREADS * i)) = st[i];
    }
    // fragment of 32 rows starting at rb for k step kk (16 k values)
    __device__ static __forceinline__ bf16x8 frag(const char* lds, int rb, int kk) {
        const int l = threadIdx.x & 63;
        if (KC) {
            const int r = rb + (l & 31), ch = 2 * kk + (l >> 5);
            return *reinterpret_cast<const bf16x8*>(lds + r * 128 + ((ch ^ ((r >> 1) & 7)) << 4));
        } else {
            typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
            const int col = rb + 16 * ((l >> 4) & 1) + 4 * (l & 3);
            const int kr0 = 16 * kk + 8 * (l >> 5) + ((l & 15) >> 2);
            const int kr1 = kr0 + 4;
            const char* p0 = lds + kr0 * (ROWS * 2) + ((col * 2) ^ ((kr0 & 3) << 6));
            const char* p1 = lds + kr1 * (ROWS * 2) + ((col * 2) ^ ((kr1 & 3) << 6));
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p0);
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p1);
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    }
};

// Workgroup -> tile mapping.  Consecutive workgroup ids land on different XCDs
// (8 of them, each with its own L2), so ids are first regrouped per XCD and each
// XCD then walks a compact block of tiles, GROUP_M tile rows at a time.
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn) {
    const int nb = tiles_m * tiles_n;
    int id = blockIdx.x;
    const int per = nb >> 3;
    if (id < per * 8) id = (id & 7) * per + (id >> 3);
    constexpr int GROUP_M = 8;
    const int width = GROUP_M * tiles_n;
    const int grp = id / width;
    const int first_m = grp * GROUP_M;
    const int gsz = min(tiles_m - first_m, GROUP_M);
    const int within = id - grp * width;
    tm = first_m + within % gsz;
    tn = within / gsz;
}

template <int KIND, int BM, int BN, bool OUT_F32>
__global__ __launch_bounds__(GTHREADS) void k_gemm_bf16(const bf16_t* __restrict__ A, int lda, uint32_t a_bytes,
                                                        const bf16_t* __restrict__ B, int ldb, uint32_t b_bytes,
                                                        void* __restrict__ Cv, int ldc, const bf16_t* R, int ldr,
                                                        int M, int N, int K, int accumulate) {
    constexpr bool A_KC = (KIND != GEMM_TN);
    constexpr bool B_KC = (KIND == GEMM_NT);
    using LA = TileLoader<BM, A_KC>;
    using LB = TileLoader<BN, B_KC>;
    constexpr int TM = BM / 64, TN = BN / 64;            // 32x32 MFMA tiles per wave in m and n
    constexpr int A_BYTES = BM * GK * 2, B_BYTES = BN * GK * 2;
    extern __shared__ __attribute__((aligned(128))) char smem[];
    char* const sA0 = smem;
    char* const sB0 = smem + 2 * A_BYTES;

    int tm, tn;
    tile_of_block((M + BM - 1) / BM, (N + BN - 1) / BN, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);

    const __amdgpu_buffer_rsrc_t rsA = make_rsrc(A, a_bytes);
    const __amdgpu_buffer_rsrc_t rsB = make_rsrc(B, b_bytes);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    i32x4 stA[LA::PER_THREAD], stB[LB::PER_THREAD];
    const int nk = (K + GK - 1) / GK;
    LA::load(stA, rsA, m0, 0, lda);
    LB::load(stB, rsB, n0, 0, ldb);
    LA::store(stA, sA0);
    LB::store(stB, sB0);
    __syncthreads();
    for (int kt = 0; kt < nk; kt++) {
        const int cur = kt & 1;
        const char* cA = sA0 + cur * A_BYTES;
        const char* cB = sB0 + cur * B_BYTES;
        if (kt + 1 < nk) {
            LA::load(stA, rsA, m0, (kt + 1) * GK, lda);
            LB::load(stB, rsB, n0, (kt + 1) * GK, ldb);
        }
#pragma unroll
        for (int kk = 0; kk < GK / 16; kk++) {
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; i++) fa[i] = LA::frag(cA, wm + 32 * i, kk);
#pragma unroll
            for (int j = 0; j < TN; j++) fb[j] = LB::frag(cB, wn + 32 * j, kk);
#pragma unroll
            for (int i = 0; i < TM; i++)
#pragma unroll
                for (int j = 0; j < TN; j++)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            LA::store(stA, sA0 + (cur ^ 1) * A_BYTES);
            LB::store(stB, sB0 + (cur ^ 1) * B_BYTES);
        }
        __syncthreads();
    }

    // epilogue: lane owns row m = .. + (lane & 31); register 4g+e holds column n = .. + 8g + 4(lane>>5) + e
    const int hf = lane >> 5;
#pragma unroll
    for (int i = 0; i < TM; i++) {
        const int m = m0 + wm + 32 * i + (lane & 31);
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < TN; j++) {
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int n = n0 + wn + 32 * j + 8 * g + 4 * hf;
                if (n >= N) continue;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] = acc[i][j][4 * g + e];
                if (OUT_F32) {
                    float* c = reinterpret_cast<float*>(Cv) + (size_t)m * ldc + n;
                    if (accumulate) {
                        const float4 old = *reinterpret_cast<const float4*>(c);
                        v[0] += old.x; v[1] += old.y; v[2] += old.z; v[3] += old.w;
                    }
                    *reinterpret_cast<float4*>(c) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
                    if (R) {
                        const uint2 rr = *reinterpret_cast<const uint2*>(R + (size_t)m * ldr + n);
                        v[0] += lo_bf(rr.x); v[1] += hi_bf(rr.x); v[2] += lo_bf(rr.y); v[3] += hi_bf(rr.y);
                    }
                    uint2 o;
                    o.x = pack_bf2(v[0], v[1]);
                    o.y = pack_bf2(v[2], v[3]);
                    *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(Cv) + (size_t)m * ldc + n) = o;
                }
            }
        }
    }
}

template <int KIND, int BM, int BN, bool OUT_F32>
static hipError_t launch(const GemmDesc& g, uint32_t a_bytes, uint32_t b_bytes, hipStream_t st) {
    constexpr int LDS = 2 * (BM + BN) * GK * 2;
    static bool attr_set = false;
    auto kern = k_gemm_bf16<KIND, BM, BN, OUT_F32>;
    if (LDS > 48 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
    kern<<<tiles, GTHREADS, LDS, st>>>((const bf16_t*)g.A, g.lda, a_bytes, (const bf16_t*)g.B, g.ldb, b_bytes, g.C, g.ldc,
                                       (const bf16_t*)g.R, g.ldr, g.M, g.N, g.K, g.accumulate);
    return hipGetLastError();
}

template <int KIND, bool OUT_F32>
static hipError_t pick_tile(const GemmDesc& g, uint32_t a_bytes, uint32_t b_bytes, hipStream_t st) {
    // 256x256 tiles when they fill the 256 CUs at least once, 128x128 otherwise
    const long big = (long)((g.M + 255) / 256) * ((g.N + 255) / 256);
    if (big >= 160) return launch<KIND, 256, 256, OUT_F32>(g, a_bytes, b_bytes, st);
    return launch<KIND, 128, 128, OUT_F32>(g, a_bytes, b_bytes, st);
}

hipError_t gemm_bf16(const GemmDesc& g, hipStream_t st) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipSuccess;
    // extent in bytes of each operand as laid out in memory (rows x ld), for the buffer bounds
    const long a_rows = (g.kind == GEMM_TN) ? g.K : g.M, a_cols = (g.kind == GEMM_TN) ? g.M : g.K;
    const long b_rows = (g.kind == GEMM_NT) ? g.N : g.K, b_cols = (g.kind == GEMM_NT) ? g.K : g.N;
    const long a_bytes = ((a_rows - 1) * g.lda + a_cols) * 2, b_bytes = ((b_rows - 1) * g.ldb + b_cols) * 2;
    if (a_bytes >= (1L << 32) - (1L << 25) || b_bytes >= (1L << 32) - (1L << 25)) return hipErrorInvalidValue;
    if (g.lda > 65535 || g.ldb > 65535) return hipErrorInvalidValue;
    // activations come out in bf16 (NT, NN), parameter gradients in fp32 (TN)
    if ((g.out_f32 != 0) != (g.kind == GEMM_TN) || (g.out_f32 && g.R)) return hipErrorInvalidValue;
    switch (g.kind) {
        case GEMM_NT: return pick_tile<GEMM_NT, false>(g, (uint32_t)a_bytes, (uint32_t)b_bytes, st);
        case GEMM_NN: return pick_tile<GEMM_NN, false>(g, (uint32_t)a_bytes, (uint32_t)b_bytes, st);
        case GEMM_TN: return pick_tile<GEMM_TN, true>(g, (uint32_t)a_bytes, (uint32_t)b_bytes, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace hh
