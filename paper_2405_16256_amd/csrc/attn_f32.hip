// fp32 causal attention for the fp32 reference-precision path (small shapes).
// One wave per query row (forward, dq) or per key row (dk, dv): lanes span keys
// (resp. queries) for the scores and span head channels for the weighted sums.
// Deterministic: no atomics.
#include "common.h"
#include "kernels.h"

namespace hh {

constexpr int AW = 4;  // waves per workgroup

__device__ __forceinline__ float dot_row(const float* __restrict__ a_lds, const float* __restrict__ row, int d) {
    float acc = 0.f;
    for (int i = 0; i < d; i += 4) {
        const float4 r = *reinterpret_cast<const float4*>(row + i);
        acc = fmaf(a_lds[i], r.x, acc); acc = fmaf(a_lds[i + 1], r.y, acc);
        acc = fmaf(a_lds[i + 2], r.z, acc); acc = fmaf(a_lds[i + 3], r.w, acc);
    }
    return acc;
}

__global__ __launch_bounds__(AW* WAVE) void k_attn_f32_fwd(const float* __restrict__ qkv, int ld, float* __restrict__ o,
                                                           float* __restrict__ lse, int B, int S, int nh, int nkv, int d) {
    __shared__ float qs[AW][128];
    const int wv = threadIdx.x / WAVE, lane = threadIdx.x % WAVE;
    const long w = (long)blockIdx.x * AW + wv;
    if (w >= (long)B * nh * S) return;  // whole wave leaves together; no block-wide barrier below
    const int s = (int)(w % S), h = (int)((w / S) % nh), b = (int)(w / ((long)S * nh));
    const int A = nh * d;
    const float* qrow = qkv + ((size_t)b * S + s) * ld + h * d;
    const float* kb = qkv + (size_t)b * S * ld + A + (h / (nh / nkv)) * d;   // the query head's key/value head
    const float* vb = kb + nkv * d;
    for (int i = lane; i < d; i += WAVE) qs[wv][i] = qrow[i];
    __builtin_amdgcn_wave_barrier();
    const float scale = 1.0f / sqrtf((float)d);
    float m = -INFINITY, l = 0.f, acc0 = 0.f, acc1 = 0.f;
    for (int t0 = 0; t0 <= s; t0 += WAVE) {
        const int t = t0 + lane;
        float z = -INFINITY;
        if (t <= s) z = dot_row(qs[wv], kb + (size_t)t * ld, d) * scale;
        const float mn = fmaxf(m, wave_max(z));
        const float alpha = expf(m - mn);
        const float p = (t <= s) ? expf(z - mn) : 0.f;
        l = l * alpha + wave_sum(p);
        acc0 *= alpha; acc1 *= alpha;
        const int nk = min(WAVE, s - t0 + 1);
        for (int j = 0; j < nk; j++) {
            const float pj = __shfl(p, j, WAVE);
            const float* vr = vb + (size_t)(t0 + j) * ld;
            if (lane < d) acc0 = fmaf(pj, vr[lane], acc0);
            if (lane + WAVE < d) acc1 = fmaf(pj, vr[lane + WAVE], acc1);
        }
        m = mn;
    }
    float* orow = o + ((size_t)b * S + s) * A + h * d;
    if (lane < d) orow[lane] = acc0 / l;
    if (lane + WAVE < d) orow[lane + WAVE] = acc1 / l;
    if (lane == 0) lse[((size_t)b * nh + h) * S + s] = m + logf(l);
}

// Per query row: D = <do, o>, and dq = sum_t dZ[s,t] k[t] / sqrt(d).
__global__ __launch_bounds__(AW* WAVE) void k_attn_f32_bwd_q(const float* __restrict__ qkv, int ld,
                                                             const float* __restrict__ o, const float* __restrict__ dout,
                                                             const float* __restrict__ lse, float* __restrict__ dvec,
                                                             float* __restrict__ dqkv, int B, int S, int nh, int nkv, int d) {
    __shared__ float qs[AW][128];
    __shared__ float dos[AW][128];
    const int wv = threadIdx.x / WAVE, lane = threadIdx.x % WAVE;
    const long w = (long)blockIdx.x * AW + wv;
    if (w >= (long)B * nh * S) return;
    const int s = (int)(w % S), h = (int)((w / S) % nh), b = (int)(w / ((long)S * nh));
    const int A = nh * d;
    const size_t tok = (size_t)b * S + s;
    const float* qrow = qkv + tok * ld + h * d;
    const float* kb = qkv + (size_t)b * S * ld + A + (h / (nh / nkv)) * d;
    const float* vb = kb + nkv * d;
    const float* dorow = dout + tok * A + h * d;
    const float* orow = o + tok * A + h * d;
    float dd = 0.f;
    for (int i = lane; i < d; i += WAVE) {
        qs[wv][i] = qrow[i];
        const float g = dorow[i];
        dos[wv][i] = g;
        dd = fmaf(g, orow[i], dd);
    }
    const float D = wave_sum(dd);
    __builtin_amdgcn_wave_barrier();
    const float L = lse[((size_t)b * nh + h) * S + s];
    if (lane == 0) dvec[((size_t)b * nh + h) * S + s] = D;
    const float scale = 1.0f / sqrtf((float)d);
    float acc0 = 0.f, acc1 = 0.f;
    for (int t0 = 0; t0 <= s; t0 += WAVE) {
        const int t = t0 + lane;
        float dz = 0.f;
        if (t <= s) {
            const float p = expf(dot_row(qs[wv], kb + (size_t)t * ld, d) * scale - L);
            const float dp = dot_row(dos[wv], vb + (size_t)t * ld, d);
            dz = p * (dp - D);
        }
        const int nk = min(WAVE, s - t0 + 1);
        for (int j = 0; j < nk; j++) {
            const float zj = __shfl(dz, j, WAVE);
            const float* kr = kb + (size_t)(t0 + j) * ld;
            if (lane < d) acc0 = fmaf(zj, kr[lane], acc0);
            if (lane + WAVE < d) acc1 = fmaf(zj, kr[lane + WAVE], acc1);
        }
    }
    float* dq = dqkv + tok * ld + h * d;
    if (lane < d) dq[lane] = acc0 * scale;
    if (lane + WAVE < d) dq[lane + WAVE] = acc1 * scale;
}

// Per key row t of key/value head hk: dv[t] = sum over its query heads and s>=t of P[s,t] do[s];
// dk[t] = the same sum of dZ[s,t] q[s] / sqrt(d).
__global__ __launch_bounds__(AW* WAVE) void k_attn_f32_bwd_kv(const float* __restrict__ qkv, int ld,
                                                              const float* __restrict__ dout, const float* __restrict__ lse,
                                                              const float* __restrict__ dvec, float* __restrict__ dqkv,
                                                              int B, int S, int nh, int nkv, int d) {
    __shared__ float ks[AW][128];
    __shared__ float vs[AW][128];
    const int wv = threadIdx.x / WAVE, lane = threadIdx.x % WAVE;
    const long w = (long)blockIdx.x * AW + wv;
    if (w >= (long)B * nkv * S) return;
    const int t = (int)(w % S), hk = (int)((w / S) % nkv), b = (int)(w / ((long)S * nkv));
    const int A = nh * d, G = nh / nkv;
    const size_t tok = (size_t)b * S + t;
    const float* krow = qkv + tok * ld + A + hk * d;
    const float* vrow = krow + nkv * d;
    for (int i = lane; i < d; i += WAVE) { ks[wv][i] = krow[i]; vs[wv][i] = vrow[i]; }
    __builtin_amdgcn_wave_barrier();
    const float scale = 1.0f / sqrtf((float)d);
    float dk0 = 0.f, dk1 = 0.f, dv0 = 0.f, dv1 = 0.f;
    for (int g = 0; g < G; g++) {
        const int h = hk * G + g;
        const float* qb = qkv + (size_t)b * S * ld + h * d;
        const float* dob = dout + (size_t)b * S * A + h * d;
        const float* Lb = lse + ((size_t)b * nh + h) * S;
        const float* Db = dvec + ((size_t)b * nh + h) * S;
        for (int s0 = t; s0 < S; s0 += WAVE) {
            const int s = s0 + lane;
            float p = 0.f, dz = 0.f;
            if (s < S) {
                p = expf(dot_row(ks[wv], qb + (size_t)s * ld, d) * scale - Lb[s]);
                const float dp = dot_row(vs[wv], dob + (size_t)s * A, d);
                dz = p * (dp - Db[s]);
            }
            const int nq = min(WAVE, S - s0);
            for (int j = 0; j < nq; j++) {
                const float pj = __shfl(p, j, WAVE), zj = __shfl(dz, j, WAVE);
                const float* qr = qb + (size_t)(s0 + j) * ld;
                const float* dr = dob + (size_t)(s0 + j) * A;
                if (lane < d) { dv0 = fmaf(pj, dr[lane], dv0); dk0 = fmaf(zj, qr[lane], dk0); }
                if (lane + WAVE < d) { dv1 = fmaf(pj, dr[lane + WAVE], dv1); dk1 = fmaf(zj, qr[lane + WAVE], dk1); }
            }
        }
    }
    float* dk = dqkv + tok * ld + A + hk * d;
    float* dv = dk + nkv * d;
    if (lane < d) { dk[lane] = dk0 * scale; dv[lane] = dv0; }
    if (lane + WAVE < d) { dk[lane + WAVE] = dk1 * scale; dv[lane + WAVE] = dv1; }
}

hipError_t attn_f32_fwd(const void* qkv, int ld, void* o, float* lse, int B, int S, int nh, int nkv, int d, hipStream_t st) {
    const long rows = (long)B * nh * S;
    k_attn_f32_fwd<<<(unsigned)((rows + AW - 1) / AW), AW * WAVE, 0, st>>>((const float*)qkv, ld, (float*)o, lse, B, S, nh, nkv, d);
    return hipGetLastError();
}

hipError_t attn_f32_bwd(const void* qkv, int ld, const void* o, const void* dout, const float* lse, float* dvec,
                        void* dqkv, int B, int S, int nh, int nkv, int d, hipStream_t st) {
    const long rows = (long)B * nh * S, rows_kv = (long)B * nkv * S;
    k_attn_f32_bwd_q<<<(unsigned)((rows + AW - 1) / AW), AW * WAVE, 0, st>>>((const float*)qkv, ld, (const float*)o, (const float*)dout,
                                                                             lse, dvec, (float*)dqkv, B, S, nh, nkv, d);
    k_attn_f32_bwd_kv<<<(unsigned)((rows_kv + AW - 1) / AW), AW * WAVE, 0, st>>>((const float*)qkv, ld, (const float*)dout, lse, dvec,
                                                                                 (float*)dqkv, B, S, nh, nkv, d);
    return hipGetLastError();
}

}  // namespace hh
