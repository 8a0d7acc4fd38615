// HBM-bound kernels of the decoder layer: RMSNorm forward/backward (with the
// residual gradient folded in), rotary embedding, SwiGLU forward/backward and
// the column-sum reduction for the gain gradients.  All global accesses are
// 16-byte vectors along the contiguous feature dimension; math is fp32.
#include "common.h"
#include "kernels.h"

namespace hh {

constexpr int TPB = 256;
constexpr int NWAVES = TPB / WAVE;

// ------------------------------------------------------------------ RMSNorm
// A row of up to RC * TPB * V elements stays in registers between the reduction pass and the
// output pass (RC raw 16-byte vectors per thread); longer rows are re-read (from L2).
constexpr int RC = 6;

template <typename T>
__global__ __launch_bounds__(TPB) void k_rmsnorm_fwd(const T* __restrict__ x, const T* __restrict__ g,
                                                     T* __restrict__ xn, float* __restrict__ r, int H, float eps) {
    constexpr int V = Vec<T>::N;
    typedef typename Vec<T>::Raw Raw;
    __shared__ float red[NWAVES];
    const size_t base = (size_t)blockIdx.x * H;
    const bool cached = H <= RC * TPB * V;
    Raw keep[RC];
    float ss = 0.f;
    if (cached) {
#pragma unroll
        for (int i = 0; i < RC; i++) {
            const int c = (threadIdx.x + i * TPB) * V;
            if (c < H) {
                keep[i] = Vec<T>::raw(x + base + c);
                float f[V];
                Vec<T>::widen(keep[i], f);
#pragma unroll
                for (int e = 0; e < V; e++) ss += f[e] * f[e];
            }
        }
    } else {
        for (int c = threadIdx.x * V; c < H; c += TPB * V) {
            float f[V];
            Vec<T>::load(x + base + c, f);
#pragma unroll
            for (int e = 0; e < V; e++) ss += f[e] * f[e];
        }
    }
    ss = block_sum<NWAVES>(ss, red);
    const float rs = 1.0f / sqrtf(ss / (float)H + eps);
    if (threadIdx.x == 0) r[blockIdx.x] = rs;
    if (cached) {
#pragma unroll
        for (int i = 0; i < RC; i++) {
            const int c = (threadIdx.x + i * TPB) * V;
            if (c < H) {
                float f[V], gg[V];
                Vec<T>::widen(keep[i], f);
                Vec<T>::load(g + c, gg);
#pragma unroll
                for (int e = 0; e < V; e++) f[e] = f[e] * rs * gg[e];
                Vec<T>::store(xn + base + c, f);
            }
        }
    } else {
        for (int c = threadIdx.x * V; c < H; c += TPB * V) {
            float f[V], gg[V];
            Vec<T>::load(x + base + c, f);
            Vec<T>::load(g + c, gg);
#pragma unroll
            for (int e = 0; e < V; e++) f[e] = f[e] * rs * gg[e];
            Vec<T>::store(xn + base + c, f);
        }
    }
}

// One workgroup walks `rpb` consecutive rows.  Column j is always handled by the
// same thread, so the per-column sums of dxn*u live in LDS without atomics.
template <typename T>
__global__ __launch_bounds__(TPB) void k_rmsnorm_bwd(const T* __restrict__ dxn, const T* __restrict__ x,
                                                     const float* __restrict__ r, const T* __restrict__ g,
                                                     const T* __restrict__ dres, T* __restrict__ dx,
                                                     float* __restrict__ partial, int T_rows, int H, int rpb) {
    constexpr int V = Vec<T>::N;
    typedef typename Vec<T>::Raw Raw;
    extern __shared__ float colacc[];  // [H]
    __shared__ float red[NWAVES];
    for (int c = threadIdx.x * V; c < H; c += TPB * V)
#pragma unroll
        for (int e = 0; e < V; e++) colacc[c + e] = 0.f;
    const int row0 = blockIdx.x * rpb;
    const int row1 = min(T_rows, row0 + rpb);
    const float invH = 1.0f / (float)H;
    const bool cached = H <= RC * TPB * V;
    for (int row = row0; row < row1; row++) {
        const size_t base = (size_t)row * H;
        const float rs = r[row];
        float s = 0.f;
        if (cached) {
            Raw kd[RC], kx[RC];
#pragma unroll
            for (int i = 0; i < RC; i++) {
                const int c = (threadIdx.x + i * TPB) * V;
                if (c < H) {
                    kd[i] = Vec<T>::raw(dxn + base + c);
                    kx[i] = Vec<T>::raw(x + base + c);
                    float d[V], xx[V], gg[V];
                    Vec<T>::widen(kd[i], d);
                    Vec<T>::widen(kx[i], xx);
                    Vec<T>::load(g + c, gg);
#pragma unroll
                    for (int e = 0; e < V; e++) s += d[e] * gg[e] * xx[e];
                }
            }
            const float c1 = block_sum<NWAVES>(s, red) * rs * invH;  // mean_j(w_j u_j)
#pragma unroll
            for (int i = 0; i < RC; i++) {
                const int c = (threadIdx.x + i * TPB) * V;
                if (c < H) {
                    float d[V], xx[V], gg[V], rr[V], o[V];
                    Vec<T>::widen(kd[i], d);
                    Vec<T>::widen(kx[i], xx);
                    Vec<T>::load(g + c, gg);
                    Vec<T>::load(dres + base + c, rr);
#pragma unroll
                    for (int e = 0; e < V; e++) {
                        const float u = xx[e] * rs;
                        colacc[c + e] += d[e] * u;
                        o[e] = rr[e] + rs * (d[e] * gg[e] - u * c1);
                    }
                    Vec<T>::store(dx + base + c, o);
                }
            }
        } else {
            for (int c = threadIdx.x * V; c < H; c += TPB * V) {
                float d[V], xx[V], gg[V];
                Vec<T>::load(dxn + base + c, d);
                Vec<T>::load(x + base + c, xx);
                Vec<T>::load(g + c, gg);
#pragma unroll
                for (int e = 0; e < V; e++) s += d[e] * gg[e] * xx[e];
            }
            const float c1 = block_sum<NWAVES>(s, red) * rs * invH;
            for (int c = threadIdx.x * V; c < H; c += TPB * V) {
                float d[V], xx[V], gg[V], rr[V], o[V];
                Vec<T>::load(dxn + base + c, d);
                Vec<T>::load(x + base + c, xx);
                Vec<T>::load(g + c, gg);
                Vec<T>::load(dres + base + c, rr);
#pragma unroll
                for (int e = 0; e < V; e++) {
                    const float u = xx[e] * rs;
                    colacc[c + e] += d[e] * u;
                    o[e] = rr[e] + rs * (d[e] * gg[e] - u * c1);
                }
                Vec<T>::store(dx + base + c, o);
            }
        }
    }
    float* out = partial + (size_t)blockIdx.x * H;
    for (int c = threadIdx.x * V; c < H; c += TPB * V)
#pragma unroll
        for (int e = 0; e < V; e++) out[c + e] = colacc[c + e];
}

// out[j] (=|+=) sum_b partial[b][j].  A workgroup covers 256 columns (one float4 per thread column
// group) with 4 row groups that are combined through LDS in a fixed order.
__global__ __launch_bounds__(TPB) void k_colsum_reduce(const float* __restrict__ partial, int nblk, int H,
                                                       float* __restrict__ out, int accumulate) {
    __shared__ float4 red[NWAVES][WAVE];
    const int cx = threadIdx.x % WAVE, ry = threadIdx.x / WAVE;
    const int col = (blockIdx.x * WAVE + cx) * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (col < H) {
        const float* p = partial + col;
#pragma unroll 8
        for (int b = ry; b < nblk; b += NWAVES) {
            const float4 v = *reinterpret_cast<const float4*>(p + (size_t)b * H);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
    }
    red[ry][cx] = s;
    __syncthreads();
    if (ry == 0 && col < H) {
        float4 t = red[0][cx];
#pragma unroll
        for (int i = 1; i < NWAVES; i++) { t.x += red[i][cx].x; t.y += red[i][cx].y; t.z += red[i][cx].z; t.w += red[i][cx].w; }
        float4* o = reinterpret_cast<float4*>(out + col);
        if (accumulate) { const float4 old = *o; t.x += old.x; t.y += old.y; t.z += old.z; t.w += old.w; }
        *o = t;
    }
}

// --------------------------------------------------------------------- RoPE
// One thread rotates V pairs (i, i + d/2) of one of the nrot heads that start at column 0 of a token's row
// (the query heads followed by the key heads).
template <typename T>
__global__ __launch_bounds__(TPB) void k_rope(T* __restrict__ qkv, int ld, int Ttok, int S, int nrot, int d,
                                              const float* __restrict__ table, int table_seq, float sin_sign) {
    constexpr int V = Vec<T>::N;
    const int half = d / 2;
    const int vph = half / V;               // vectors per head-half
    const long total = (long)Ttok * nrot * vph;
    const long idx = (long)blockIdx.x * TPB + threadIdx.x;
    if (idx >= total) return;
    const int iv = (int)(idx % vph);
    long rest = idx / vph;
    const int head = (int)(rest % nrot);
    const int t = (int)(rest / nrot);
    const int pos = t % S;
    T* p = qkv + (size_t)t * ld + (size_t)head * d + iv * V;
    const float* cs = table + ((size_t)pos * half + iv * V);
    const float* sn = cs + (size_t)table_seq * half;
    float a[V], b[V], oa[V], ob[V];
    Vec<T>::load(p, a);
    Vec<T>::load(p + half, b);
#pragma unroll
    for (int e = 0; e < V; e++) {
        const float c = cs[e], s = sin_sign * sn[e];
        oa[e] = a[e] * c - b[e] * s;
        ob[e] = b[e] * c + a[e] * s;
    }
    Vec<T>::store(p, oa);
    Vec<T>::store(p + half, ob);
}

// ------------------------------------------------------------------- SwiGLU
template <typename T>
__global__ __launch_bounds__(TPB) void k_swiglu_fwd(const T* __restrict__ gu, T* __restrict__ m, int Ttok, int F) {
    constexpr int V = Vec<T>::N;
    const int vpr = F / V;
    const long idx = (long)blockIdx.x * TPB + threadIdx.x;
    if (idx >= (long)Ttok * vpr) return;
    const int t = (int)(idx / vpr), c = (int)(idx % vpr) * V;
    float gt[V], u[V], o[V];
    Vec<T>::load(gu + (size_t)t * 2 * F + c, gt);
    Vec<T>::load(gu + (size_t)t * 2 * F + F + c, u);
#pragma unroll
    for (int e = 0; e < V; e++) o[e] = gt[e] / (1.0f + expf(-gt[e])) * u[e];
    Vec<T>::store(m + (size_t)t * F + c, o);
}

template <typename T>
__global__ __launch_bounds__(TPB) void k_swiglu_bwd(const T* __restrict__ dm, const T* __restrict__ gu,
                                                    T* __restrict__ dgu, T* __restrict__ m, int Ttok, int F) {
    constexpr int V = Vec<T>::N;
    const int vpr = F / V;
    const long idx = (long)blockIdx.x * TPB + threadIdx.x;
    if (idx >= (long)Ttok * vpr) return;
    const int t = (int)(idx / vpr), c = (int)(idx % vpr) * V;
    float gt[V], u[V], d[V], og[V], ou[V], om[V];
    Vec<T>::load(gu + (size_t)t * 2 * F + c, gt);
    Vec<T>::load(gu + (size_t)t * 2 * F + F + c, u);
    Vec<T>::load(dm + (size_t)t * F + c, d);
#pragma unroll
    for (int e = 0; e < V; e++) {
        const float sg = 1.0f / (1.0f + expf(-gt[e]));
        const float sl = gt[e] * sg;
        om[e] = sl * u[e];
        og[e] = d[e] * u[e] * sg * (1.0f + gt[e] * (1.0f - sg));
        ou[e] = d[e] * sl;
    }
    Vec<T>::store(dgu + (size_t)t * 2 * F + c, og);
    Vec<T>::store(dgu + (size_t)t * 2 * F + F + c, ou);
    Vec<T>::store(m + (size_t)t * F + c, om);
}

// ---------------------------------------------------------------- launchers
static inline unsigned nblocks(long n) { return (unsigned)((n + TPB - 1) / TPB); }

hipError_t rmsnorm_fwd(int dtype, const void* x, const void* g, void* xn, float* r, int T, int H, float eps,
                       hipStream_t st) {
    if (dtype == DT_BF16)
        k_rmsnorm_fwd<bf16_t><<<T, TPB, 0, st>>>((const bf16_t*)x, (const bf16_t*)g, (bf16_t*)xn, r, H, eps);
    else
        k_rmsnorm_fwd<float><<<T, TPB, 0, st>>>((const float*)x, (const float*)g, (float*)xn, r, H, eps);
    return hipGetLastError();
}

// Rows of exactly NV * TPB * V elements: the three input rows of row r + 1 are requested before row r is
// reduced and written, each in its own registers, so the memory queue never drains between rows.  The one
// barrier per row waits for LDS only (a full workgroup fence would also wait for the loads in flight).
__device__ __forceinline__ void keep_raw(uint4& v) { asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w)); }
__device__ __forceinline__ void keep_raw(float4& v) { asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w)); }

template <typename T, int NV>
__global__ __launch_bounds__(TPB, 2) void k_rmsnorm_bwd_rows(const T* __restrict__ dxn, const T* __restrict__ x,
                                                          const float* __restrict__ r, const T* __restrict__ g,
                                                          const T* __restrict__ dres, T* __restrict__ dx,
                                                          float* __restrict__ partial, int T_rows, int rpb) {
    constexpr int V = Vec<T>::N;
    constexpr int H = NV * TPB * V;
    typedef typename Vec<T>::Raw Raw;
    extern __shared__ float colacc[];  // [H]
    __shared__ float red[2][NWAVES];
    struct Row { Raw d[NV], x[NV], res[NV]; float rs; };
    auto fetch = [&](Row& w, int row) {
        const size_t base = (size_t)row * H;
#pragma unroll
        for (int i = 0; i < NV; i++) {
            const int c = (threadIdx.x + i * TPB) * V;
            w.d[i] = Vec<T>::raw(dxn + base + c);
            w.x[i] = Vec<T>::raw(x + base + c);
            w.res[i] = Vec<T>::raw(dres + base + c);
        }
        w.rs = r[row];
    };
    Raw gain[NV];
#pragma unroll
    for (int i = 0; i < NV; i++) {
        const int c = (threadIdx.x + i * TPB) * V;
        gain[i] = Vec<T>::raw(g + c);
#pragma unroll
        for (int e = 0; e < V; e++) colacc[c + e] = 0.f;   // only this thread ever touches these columns
    }
    const int row0 = blockIdx.x * rpb;
    const int row1 = min(T_rows, row0 + rpb);
    const float invH = 1.0f / (float)H;
    const int wave = threadIdx.x / WAVE, lane = threadIdx.x & (WAVE - 1);
    auto finish = [&](Row& w, int row) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < NV; i++) {
            float d[V], xx[V], gg[V];
            Vec<T>::widen(w.d[i], d);
            Vec<T>::widen(w.x[i], xx);
            Vec<T>::widen(gain[i], gg);
#pragma unroll
            for (int e = 0; e < V; e++) s += d[e] * gg[e] * xx[e];
        }
        s = wave_sum(s);
        float* rd = red[row & 1];      // the other parity's readers are a barrier behind at most
        if (lane == 0) rd[wave] = s;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        float tot = 0.f;
#pragma unroll
        for (int i = 0; i < NWAVES; i++) tot += rd[i];
        // the raw rows are unpacked a second time below: keeping the fp32 copies of the first pass alive
        // across the barrier would double the registers a row takes
#pragma unroll
        for (int i = 0; i < NV; i++) { keep_raw(w.d[i]); keep_raw(w.x[i]); }
        const float rs = w.rs;
        const float c1 = tot * rs * invH;  // mean_j(w_j u_j)
        const size_t base = (size_t)row * H;
#pragma unroll
        for (int i = 0; i < NV; i++) {
            const int c = (threadIdx.x + i * TPB) * V;
            float d[V], xx[V], gg[V], rr[V], o[V];
            Vec<T>::widen(w.d[i], d);
            Vec<T>::widen(w.x[i], xx);
            Vec<T>::widen(gain[i], gg);
            Vec<T>::widen(w.res[i], rr);
#pragma unroll
            for (int e = 0; e < V; e++) {
                const float u = xx[e] * rs;
                colacc[c + e] += d[e] * u;
                o[e] = rr[e] + rs * (d[e] * gg[e] - u * c1);
            }
            Vec<T>::store(dx + base + c, o);
        }
    };
    if (row0 >= row1) return;
    // fetches past the block's last row re-read that row (in bounds, unused): no branch around a request
    const int last = row1 - 1;
    Row a, b;
    fetch(a, row0);
    for (int row = row0; row < row1; row += 2) {
        fetch(b, min(row + 1, last));
        finish(a, row);
        fetch(a, min(row + 2, last));
        if (row + 1 < row1) finish(b, row + 1);
    }
#pragma unroll
    for (int i = 0; i < NV; i++) {
        const int c = (threadIdx.x + i * TPB) * V;
#pragma unroll
        for (int e = 0; e < V; e++) partial[(size_t)blockIdx.x * H + c + e] = colacc[c + e];
    }
}

template <typename T, int NV>
static hipError_t launch_rmsnorm_bwd_rows(const void* dxn, const void* x, const float* r, const void* g, const void* dres,
                                          void* dx, float* partial, int T_rows, int rpb, int nblk, hipStream_t st) {
    constexpr int lds = NV * TPB * Vec<T>::N * (int)sizeof(float);
    static std::atomic<uint64_t> lds_ok{0};
    const hipError_t e = allow_lds((const void*)k_rmsnorm_bwd_rows<T, NV>, lds, lds_ok);
    if (e != hipSuccess) return e;
    k_rmsnorm_bwd_rows<T, NV><<<nblk, TPB, lds, st>>>((const T*)dxn, (const T*)x, r, (const T*)g, (const T*)dres, (T*)dx,
                                                      partial, T_rows, rpb);
    return hipGetLastError();
}

static inline int rms_rows_per_block(int T) {
    int rpb = 8;
    while ((T + rpb - 1) / rpb > 256) rpb *= 2;
    return rpb;
}
int rmsnorm_bwd_blocks(int T) {
    const int rpb = rms_rows_per_block(T);
    return (T + rpb - 1) / rpb;
}

hipError_t rmsnorm_bwd(int dtype, const void* dxn, const void* x, const float* r, const void* g, const void* dres,
                       void* dx, float* partial, int T, int H, hipStream_t st) {
    const int rpb = rms_rows_per_block(T);
    const int nblk = (T + rpb - 1) / rpb;
    const size_t lds = (size_t)H * sizeof(float);
    hipError_t e;
    if (dtype == DT_BF16 && H % (TPB * 8) == 0 && H / (TPB * 8) <= RC) {
        switch (H / (TPB * 8)) {   // row length as a compile-time multiple of the workgroup's 16-byte vectors
            case 1: return launch_rmsnorm_bwd_rows<bf16_t, 1>(dxn, x, r, g, dres, dx, partial, T, rpb, nblk, st);
            case 2: return launch_rmsnorm_bwd_rows<bf16_t, 2>(dxn, x, r, g, dres, dx, partial, T, rpb, nblk, st);
            case 3: return launch_rmsnorm_bwd_rows<bf16_t, 3>(dxn, x, r, g, dres, dx, partial, T, rpb, nblk, st);
            case 4: return launch_rmsnorm_bwd_rows<bf16_t, 4>(dxn, x, r, g, dres, dx, partial, T, rpb, nblk, st);
            case 5: return launch_rmsnorm_bwd_rows<bf16_t, 5>(dxn, x, r, g, dres, dx, partial, T, rpb, nblk, st);
            default: return launch_rmsnorm_bwd_rows<bf16_t, 6>(dxn, x, r, g, dres, dx, partial, T, rpb, nblk, st);
        }
    }
    if (dtype == DT_BF16) {
        if (lds > 48 * 1024) {
            e = hipFuncSetAttribute((const void*)k_rmsnorm_bwd<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        k_rmsnorm_bwd<bf16_t><<<nblk, TPB, lds, st>>>((const bf16_t*)dxn, (const bf16_t*)x, r, (const bf16_t*)g,
                                                      (const bf16_t*)dres, (bf16_t*)dx, partial, T, H, rpb);
    } else {
        if (lds > 48 * 1024) {
            e = hipFuncSetAttribute((const void*)k_rmsnorm_bwd<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        k_rmsnorm_bwd<float><<<nblk, TPB, lds, st>>>((const float*)dxn, (const float*)x, r, (const float*)g,
                                                     (const float*)dres, (float*)dx, partial, T, H, rpb);
    }
    return hipGetLastError();
}

hipError_t colsum_reduce(const float* partial, int nblk, int H, float* out, int accumulate, hipStream_t st) {
    k_colsum_reduce<<<(H + 4 * WAVE - 1) / (4 * WAVE), TPB, 0, st>>>(partial, nblk, H, out, accumulate);
    return hipGetLastError();
}

hipError_t rope(int dtype, void* qkv, int ld, int T, int S, int nrot, int d, const float* table, int table_seq,
                int backward, hipStream_t st) {
    const float sgn = backward ? -1.0f : 1.0f;
    if (dtype == DT_BF16) {
        const long n = (long)T * nrot * (d / 2 / Vec<bf16_t>::N);
        k_rope<bf16_t><<<nblocks(n), TPB, 0, st>>>((bf16_t*)qkv, ld, T, S, nrot, d, table, table_seq, sgn);
    } else {
        const long n = (long)T * nrot * (d / 2 / Vec<float>::N);
        k_rope<float><<<nblocks(n), TPB, 0, st>>>((float*)qkv, ld, T, S, nrot, d, table, table_seq, sgn);
    }
    return hipGetLastError();
}

hipError_t swiglu_fwd(int dtype, const void* gu, void* m, int T, int F, hipStream_t st) {
    if (dtype == DT_BF16)
        k_swiglu_fwd<bf16_t><<<nblocks((long)T * (F / 8)), TPB, 0, st>>>((const bf16_t*)gu, (bf16_t*)m, T, F);
    else
        k_swiglu_fwd<float><<<nblocks((long)T * (F / 4)), TPB, 0, st>>>((const float*)gu, (float*)m, T, F);
    return hipGetLastError();
}

hipError_t swiglu_bwd(int dtype, const void* dm, const void* gu, void* dgu, void* m, int T, int F, hipStream_t st) {
    if (dtype == DT_BF16)
        k_swiglu_bwd<bf16_t><<<nblocks((long)T * (F / 8)), TPB, 0, st>>>((const bf16_t*)dm, (const bf16_t*)gu,
                                                                          (bf16_t*)dgu, (bf16_t*)m, T, F);
    else
        k_swiglu_bwd<float><<<nblocks((long)T * (F / 4)), TPB, 0, st>>>((const float*)dm, (const float*)gu,
                                                                         (float*)dgu, (float*)m, T, F);
    return hipGetLastError();
}

}  // namespace hh
