// Causal flash-style attention, forward and backward, bf16 on the gfx950 matrix
// cores.  The S x S score matrix is never written out: K/V (forward, dQ pass) or
// Q/dO (dK/dV pass) tiles of 64 rows are staged in LDS and each wave owns 32
// queries (resp. 32 keys) whose operands stay in registers.
//
// All products are computed transposed -- S^T = K Q^T, O^T = V^T P^T, ... -- so
// that the 32x32 MFMA accumulator gives every lane ONE query (forward, dQ) or
// ONE key (dK/dV) and spreads the other index over registers: the softmax
// row-reductions are then register-local plus one exchange between the two
// half-waves, and the accumulator registers, packed to bf16, are already the
// second operand of the next MFMA (a lane's 8 values for k-step kk are rows
// 16kk + 8(s/4) + 4(lane/32) + s%4 of the tile, s = 0..7).  The first operand
// of that MFMA needs the staged tile transposed; it is read with
// ds_read_b64_tr_b16 from the [row][d] layout, rows chosen to match that order.
//
// Backward is two deterministic passes (no atomics): a query-stationary pass
// for dQ and a key-stationary pass for dK, dV, both recomputing P from the
// saved log-sum-exp.  delta[s] = <dO[s], O[s]> comes from a small pre-pass.
#include "common.h"
#include "kernels.h"

namespace hh {

constexpr int ATHREADS = 256;
constexpr float LOG2E = 1.4426950408889634f;

typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

// [64][D] bf16 tile, global -> LDS, rows tok0.. of a [*, ld] buffer at column col0
template <int D, int PITCH>
__device__ __forceinline__ void load_tile64(char* lds, __amdgpu_buffer_rsrc_t rs, uint32_t tok0, int ld, int col0) {
    constexpr int CPR = D / 8;
#pragma unroll
    for (int i = 0; i < 64 * CPR / ATHREADS; i++) {
        const int c = threadIdx.x + ATHREADS * i;
        const int r = c / CPR, ch = c % CPR;
        const uint32_t off = ((tok0 + r) * (uint32_t)ld + (uint32_t)(col0 + ch * 8)) * 2u;
        const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
        *reinterpret_cast<i32x4*>(lds + r * PITCH + ch * 16) = v;
    }
}

// rows rb + (lane%32), k = 16kk + 8(lane/32) .. +7 along d
template <int PITCH>
__device__ __forceinline__ bf16x8 frag_rows(const char* lds, int rb, int kk) {
    const int l = threadIdx.x & 63;
    return *reinterpret_cast<const bf16x8*>(lds + (rb + (l & 31)) * PITCH + (16 * kk + 8 * (l >> 5)) * 2);
}

// transposed fragment: result row = tile column cb + (lane%32); the lane's 8 k values are
// tile rows 16kk + 8j + 4(lane/32) + e  (j = 0,1; e = 0..3)
template <int PITCH>
__device__ __forceinline__ bf16x8 frag_cols(const char* lds, int cb, int kk) {
    const int l = threadIdx.x & 63;
    const int row = 16 * kk + 4 * (l >> 5) + ((l & 15) >> 2);
    const int col = cb + 16 * ((l >> 4) & 1) + 4 * (l & 3);
    const char* p = lds + row * PITCH + col * 2;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p);
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + 8 * PITCH));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// accumulator registers 8*half .. 8*half+7 -> bf16 operand
__device__ __forceinline__ bf16x8 pack8(const f32x16& a, int half) {
    union { uint32_t u[4]; bf16x8 v; } r;
#pragma unroll
    for (int i = 0; i < 4; i++) r.u[i] = pack_bf2(a[8 * half + 2 * i], a[8 * half + 2 * i + 1]);
    return r.v;
}

template <int D>
__device__ __forceinline__ void load_qfrag(bf16x8 (&f)[D / 16], __amdgpu_buffer_rsrc_t rs, uint32_t tok, int ld, int col0) {
    const int l = threadIdx.x & 63;
#pragma unroll
    for (int kk = 0; kk < D / 16; kk++) {
        const uint32_t off = (tok * (uint32_t)ld + (uint32_t)(col0 + 16 * kk + 8 * (l >> 5))) * 2u;
        union { i32x4 i; bf16x8 v; } u;
        u.i = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
        f[kk] = u.v;
    }
}

// ------------------------------------------------------------------ forward
template <int D>
__global__ __launch_bounds__(ATHREADS) void k_attn_fwd(const bf16_t* __restrict__ qkv, int ld, uint32_t qkv_bytes,
                                                       bf16_t* __restrict__ o, float* __restrict__ lse, int S, int nh) {
    constexpr int PK = D * 2 + 16, PV = D * 2 + 64;
    __shared__ __attribute__((aligned(16))) char sK[64 * PK];
    __shared__ __attribute__((aligned(16))) char sV[64 * PV];
    const int qb = gridDim.x - 1 - blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int A = nh * D;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5;
    const int q0 = qb * 128 + wave * 32;
    const int query = q0 + (lane & 31);
    const uint32_t tokb = (uint32_t)b * S;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(qkv, qkv_bytes);

    bf16x8 qf[D / 16];
    load_qfrag<D>(qf, rs, tokb + query, ld, h * D);

    f32x16 oacc[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) oacc[i][r] = 0.f;
    float m = -INFINITY, lsum = 0.f;
    const float c = LOG2E / sqrtf((float)D);

    const int q_last = min(qb * 128 + 127, S - 1);
    for (int kv0 = 0; kv0 <= q_last; kv0 += 64) {
        __syncthreads();
        load_tile64<D, PK>(sK, rs, tokb + kv0, ld, A + h * D);
        load_tile64<D, PV>(sV, rs, tokb + kv0, ld, 2 * A + h * D);
        __syncthreads();
        if (kv0 > q0 + 31) continue;  // every key of the tile lies after every query of this wave
        f32x16 sacc[2];
#pragma unroll
        for (int tl = 0; tl < 2; tl++) {
#pragma unroll
            for (int r = 0; r < 16; r++) sacc[tl][r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < D / 16; kk++)
                sacc[tl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<PK>(sK, 32 * tl, kk), qf[kk], sacc[tl], 0, 0, 0);
        }
        float tmax = -INFINITY;
        const bool diag = kv0 + 63 > q0;
#pragma unroll
        for (int tl = 0; tl < 2; tl++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
                float s = sacc[tl][r] * c;
                if (diag) {
                    const int key = kv0 + 32 * tl + 8 * (r >> 2) + 4 * hf + (r & 3);
                    if (key > query) s = -INFINITY;
                }
                sacc[tl][r] = s;
                tmax = fmaxf(tmax, s);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, WAVE));
        const float mn = fmaxf(m, tmax);
        const float alpha = __builtin_amdgcn_exp2f(m - mn);
        float psum = 0.f;
#pragma unroll
        for (int tl = 0; tl < 2; tl++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const float p = __builtin_amdgcn_exp2f(sacc[tl][r] - mn);
                sacc[tl][r] = p;
                psum += p;
            }
        lsum = lsum * alpha + psum;
        m = mn;
#pragma unroll
        for (int i = 0; i < D / 32; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) oacc[i][r] *= alpha;
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
            const bf16x8 pf = pack8(sacc[kk >> 1], kk & 1);
#pragma unroll
            for (int dt = 0; dt < D / 32; dt++)
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<PV>(sV, 32 * dt, kk), pf, oacc[dt], 0, 0, 0);
        }
    }
    lsum += __shfl_xor(lsum, 32, WAVE);
    if (query < S) {
        const float inv = 1.0f / lsum;
        bf16_t* orow = o + (size_t)(tokb + query) * A + h * D;
#pragma unroll
        for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                uint2 v;
                v.x = pack_bf2(oacc[dt][4 * g] * inv, oacc[dt][4 * g + 1] * inv);
                v.y = pack_bf2(oacc[dt][4 * g + 2] * inv, oacc[dt][4 * g + 3] * inv);
                *reinterpret_cast<uint2*>(orow + 32 * dt + 8 * g + 4 * hf) = v;
            }
        // m is in the log2 domain of the scaled scores
        if (hf == 0) lse[((size_t)b * nh + h) * S + query] = m / LOG2E + logf(lsum);
    }
}

// ----------------------------------------------------- delta = <dO, O> per row
template <int D>
__global__ __launch_bounds__(ATHREADS) void k_attn_delta(const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout,
                                                         float* __restrict__ dvec, int B, int S, int nh) {
    const long w = (long)blockIdx.x * (ATHREADS / WAVE) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (w >= (long)B * S * nh) return;
    const int h = (int)(w % nh);
    const long tok = w / nh;
    const int b = (int)(tok / S), s = (int)(tok % S);
    const size_t base = (size_t)tok * nh * D + (size_t)h * D + lane * (D / 64);
    float acc = 0.f;
    if (D == 128) {
        const uint32_t a = *reinterpret_cast<const uint32_t*>(o + base), g = *reinterpret_cast<const uint32_t*>(dout + base);
        acc = lo_bf(a) * lo_bf(g) + hi_bf(a) * hi_bf(g);
    } else {
        acc = bf2f(o[base]) * bf2f(dout[base]);
    }
    acc = wave_sum(acc);
    if (lane == 0) dvec[((size_t)b * nh + h) * S + s] = acc;
}

// --------------------------------------------------------------- backward: dQ
template <int D>
__global__ __launch_bounds__(ATHREADS) void k_attn_bwd_dq(const bf16_t* __restrict__ qkv, int ld, uint32_t qkv_bytes,
                                                          const bf16_t* __restrict__ dout, uint32_t do_bytes,
                                                          const float* __restrict__ lse, const float* __restrict__ dvec,
                                                          bf16_t* __restrict__ dqkv, int S, int nh) {
    constexpr int PK = D * 2 + 16, PV = D * 2 + 16;
    __shared__ __attribute__((aligned(16))) char sK[64 * PK];
    __shared__ __attribute__((aligned(16))) char sV[64 * PV];
    const int qb = gridDim.x - 1 - blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int A = nh * D;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5;
    const int q0 = qb * 128 + wave * 32;
    const int query = q0 + (lane & 31);
    const uint32_t tokb = (uint32_t)b * S;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(qkv, qkv_bytes);
    const __amdgpu_buffer_rsrc_t rsdo = make_rsrc(dout, do_bytes);

    bf16x8 qf[D / 16], dof[D / 16];
    load_qfrag<D>(qf, rs, tokb + query, ld, h * D);
    load_qfrag<D>(dof, rsdo, tokb + query, A, h * D);
    const float sc = 1.0f / sqrtf((float)D);
    const float c = LOG2E * sc;
    float L = 0.f, dl = 0.f;
    if (query < S) {
        L = lse[((size_t)b * nh + h) * S + query] * LOG2E;
        dl = dvec[((size_t)b * nh + h) * S + query];
    }
    f32x16 dq[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) dq[i][r] = 0.f;

    const int q_last = min(qb * 128 + 127, S - 1);
    for (int kv0 = 0; kv0 <= q_last; kv0 += 64) {
        __syncthreads();
        load_tile64<D, PK>(sK, rs, tokb + kv0, ld, A + h * D);
        load_tile64<D, PV>(sV, rs, tokb + kv0, ld, 2 * A + h * D);
        __syncthreads();
        if (kv0 > q0 + 31) continue;
        f32x16 sacc[2], pacc[2];
#pragma unroll
        for (int tl = 0; tl < 2; tl++) {
#pragma unroll
            for (int r = 0; r < 16; r++) { sacc[tl][r] = 0.f; pacc[tl][r] = 0.f; }
#pragma unroll
            for (int kk = 0; kk < D / 16; kk++) {
                sacc[tl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<PK>(sK, 32 * tl, kk), qf[kk], sacc[tl], 0, 0, 0);
                pacc[tl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<PV>(sV, 32 * tl, kk), dof[kk], pacc[tl], 0, 0, 0);
            }
        }
        const bool diag = kv0 + 63 > q0;
#pragma unroll
        for (int tl = 0; tl < 2; tl++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
                float p = __builtin_amdgcn_exp2f(sacc[tl][r] * c - L);
                if (diag) {
                    const int key = kv0 + 32 * tl + 8 * (r >> 2) + 4 * hf + (r & 3);
                    if (key > query) p = 0.f;
                }
                sacc[tl][r] = p * (pacc[tl][r] - dl);  // dS^T (before the 1/sqrt(d) factor)
            }
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
            const bf16x8 sf = pack8(sacc[kk >> 1], kk & 1);
#pragma unroll
            for (int dt = 0; dt < D / 32; dt++)
                dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<PK>(sK, 32 * dt, kk), sf, dq[dt], 0, 0, 0);
        }
    }
    if (query < S) {
        bf16_t* row = dqkv + (size_t)(tokb + query) * ld + h * D;
#pragma unroll
        for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                uint2 v;
                v.x = pack_bf2(dq[dt][4 * g] * sc, dq[dt][4 * g + 1] * sc);
                v.y = pack_bf2(dq[dt][4 * g + 2] * sc, dq[dt][4 * g + 3] * sc);
                *reinterpret_cast<uint2*>(row + 32 * dt + 8 * g + 4 * hf) = v;
            }
    }
}

// ----------------------------------------------------------- backward: dK, dV
template <int D>
__global__ __launch_bounds__(ATHREADS) void k_attn_bwd_dkv(const bf16_t* __restrict__ qkv, int ld, uint32_t qkv_bytes,
                                                           const bf16_t* __restrict__ dout, uint32_t do_bytes,
                                                           const float* __restrict__ lse, const float* __restrict__ dvec,
                                                           bf16_t* __restrict__ dqkv, int S, int nh) {
    constexpr int PQ = D * 2 + 16;
    __shared__ __attribute__((aligned(16))) char sQ[64 * PQ];
    __shared__ __attribute__((aligned(16))) char sO[64 * PQ];
    __shared__ __attribute__((aligned(16))) float sL[64];
    __shared__ __attribute__((aligned(16))) float sD[64];
    const int kb = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int A = nh * D;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5;
    const int k0 = kb * 128 + wave * 32;
    const int key = k0 + (lane & 31);
    const uint32_t tokb = (uint32_t)b * S;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(qkv, qkv_bytes);
    const __amdgpu_buffer_rsrc_t rsdo = make_rsrc(dout, do_bytes);

    bf16x8 kf[D / 16], vf[D / 16];
    load_qfrag<D>(kf, rs, tokb + key, ld, A + h * D);
    load_qfrag<D>(vf, rs, tokb + key, ld, 2 * A + h * D);
    const float sc = 1.0f / sqrtf((float)D);
    const float c = LOG2E * sc;
    f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) { dk[i][r] = 0.f; dv[i][r] = 0.f; }

    for (int qt = kb * 128; qt < S; qt += 64) {
        __syncthreads();
        load_tile64<D, PQ>(sQ, rs, tokb + qt, ld, h * D);
        load_tile64<D, PQ>(sO, rsdo, tokb + qt, A, h * D);
        if (threadIdx.x < 64) {
            const int q = qt + threadIdx.x;
            const bool ok = q < S;
            sL[threadIdx.x] = ok ? lse[((size_t)b * nh + h) * S + q] * LOG2E : 0.f;
            sD[threadIdx.x] = ok ? dvec[((size_t)b * nh + h) * S + q] : 0.f;
        }
        __syncthreads();
        if (qt + 63 < k0) continue;  // every query of the tile precedes every key of this wave
        f32x16 sacc[2], pacc[2];
#pragma unroll
        for (int tl = 0; tl < 2; tl++) {
#pragma unroll
            for (int r = 0; r < 16; r++) { sacc[tl][r] = 0.f; pacc[tl][r] = 0.f; }
#pragma unroll
            for (int kk = 0; kk < D / 16; kk++) {
                sacc[tl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<PQ>(sQ, 32 * tl, kk), kf[kk], sacc[tl], 0, 0, 0);
                pacc[tl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<PQ>(sO, 32 * tl, kk), vf[kk], pacc[tl], 0, 0, 0);
            }
        }
        const bool edge = (qt < k0 + 31) || (qt + 63 >= S);
#pragma unroll
        for (int tl = 0; tl < 2; tl++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int qi = 32 * tl + 8 * g + 4 * hf;
                const float4 l4 = *reinterpret_cast<const float4*>(&sL[qi]);
                const float4 d4 = *reinterpret_cast<const float4*>(&sD[qi]);
                const float ls[4] = {l4.x, l4.y, l4.z, l4.w}, ds[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const int r = 4 * g + e;
                    float p = __builtin_amdgcn_exp2f(sacc[tl][r] * c - ls[e]);
                    if (edge) {
                        const int q = qt + qi + e;
                        if (key > q || q >= S) p = 0.f;
                    }
                    sacc[tl][r] = p;
                    pacc[tl][r] = p * (pacc[tl][r] - ds[e]);
                }
            }
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
            const bf16x8 pf = pack8(sacc[kk >> 1], kk & 1);
            const bf16x8 sf = pack8(pacc[kk >> 1], kk & 1);
#pragma unroll
            for (int dt = 0; dt < D / 32; dt++) {
                dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<PQ>(sO, 32 * dt, kk), pf, dv[dt], 0, 0, 0);
                dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<PQ>(sQ, 32 * dt, kk), sf, dk[dt], 0, 0, 0);
            }
        }
    }
    if (key < S) {
        bf16_t* krow = dqkv + (size_t)(tokb + key) * ld + A + h * D;
        bf16_t* vrow = krow + A;
#pragma unroll
        for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                uint2 v;
                v.x = pack_bf2(dk[dt][4 * g] * sc, dk[dt][4 * g + 1] * sc);
                v.y = pack_bf2(dk[dt][4 * g + 2] * sc, dk[dt][4 * g + 3] * sc);
                *reinterpret_cast<uint2*>(krow + 32 * dt + 8 * g + 4 * hf) = v;
                v.x = pack_bf2(dv[dt][4 * g], dv[dt][4 * g + 1]);
                v.y = pack_bf2(dv[dt][4 * g + 2], dv[dt][4 * g + 3]);
                *reinterpret_cast<uint2*>(vrow + 32 * dt + 8 * g + 4 * hf) = v;
            }
    }
}

// ---------------------------------------------------------------- launchers
hipError_t attn_bf16_fwd(const void* qkv, int ld, void* o, float* lse, int B, int S, int nh, int d, hipStream_t st) {
    const long bytes = (long)B * S * ld * 2;
    if (bytes >= (1L << 32) - (1L << 25)) return hipErrorInvalidValue;
    dim3 grid((S + 127) / 128, nh, B);
    if (d == 128)
        k_attn_fwd<128><<<grid, ATHREADS, 0, st>>>((const bf16_t*)qkv, ld, (uint32_t)bytes, (bf16_t*)o, lse, S, nh);
    else if (d == 64)
        k_attn_fwd<64><<<grid, ATHREADS, 0, st>>>((const bf16_t*)qkv, ld, (uint32_t)bytes, (bf16_t*)o, lse, S, nh);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t attn_bf16_bwd(const void* qkv, int ld, const void* o, const void* dout, const float* lse, float* dvec,
                         void* dqkv, int B, int S, int nh, int d, hipStream_t st) {
    const long bytes = (long)B * S * ld * 2;
    const long do_bytes = (long)B * S * nh * d * 2;
    if (bytes >= (1L << 32) - (1L << 25)) return hipErrorInvalidValue;
    dim3 grid((S + 127) / 128, nh, B);
    const long rows = (long)B * S * nh;
    const unsigned nb = (unsigned)((rows + 3) / 4);
    if (d == 128) {
        k_attn_delta<128><<<nb, ATHREADS, 0, st>>>((const bf16_t*)o, (const bf16_t*)dout, dvec, B, S, nh);
        k_attn_bwd_dq<128><<<grid, ATHREADS, 0, st>>>((const bf16_t*)qkv, ld, (uint32_t)bytes, (const bf16_t*)dout,
                                                      (uint32_t)do_bytes, lse, dvec, (bf16_t*)dqkv, S, nh);
        k_attn_bwd_dkv<128><<<grid, ATHREADS, 0, st>>>((const bf16_t*)qkv, ld, (uint32_t)bytes, (const bf16_t*)dout,
                                                       (uint32_t)do_bytes, lse, dvec, (bf16_t*)dqkv, S, nh);
    } else if (d == 64) {
        k_attn_delta<64><<<nb, ATHREADS, 0, st>>>((const bf16_t*)o, (const bf16_t*)dout, dvec, B, S, nh);
        k_attn_bwd_dq<64><<<grid, ATHREADS, 0, st>>>((const bf16_t*)qkv, ld, (uint32_t)bytes, (const bf16_t*)dout,
                                                     (uint32_t)do_bytes, lse, dvec, (bf16_t*)dqkv, S, nh);
        k_attn_bwd_dkv<64><<<grid, ATHREADS, 0, st>>>((const bf16_t*)qkv, ld, (uint32_t)bytes, (const bf16_t*)dout,
                                                      (uint32_t)do_bytes, lse, dvec, (bf16_t*)dqkv, S, nh);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace hh
