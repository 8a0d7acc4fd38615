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
// saved log-sum-exp.  On large launches they are two kernels and the dQ pass forms
// delta[s] = <dO[s], O[s]> for the dK/dV pass; on launches of few workgroups, where
// each pass alone is bound by its longest job, a small kernel forms delta and one
// launch deals out the jobs of both passes together.
//
// The loops are bound by instruction issue, not by the matrix pipes, so the vector
// work per tile is kept to the softmax arithmetic itself: LDS addresses are per-lane
// tables whose tile, row-block and k-step displacements sit in the instructions'
// offset fields, the lane part of every tile-load address is computed once, and the
// causal mask is applied by a branch on the (few) tiles that touch the diagonal.
#include "common.h"
#include "kernels.h"

namespace hh {

constexpr int ATHREADS = 256;
constexpr float LOG2E = 1.4426950408889634f;

typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

// A staged tile is 64 rows x D bf16, rows contiguous (D*2 bytes), 16-byte chunks XOR-swizzled by
// the row so that both the row-wise ds_read_b128 fragments and the transposing
// ds_read_b64_tr_b16 fragments avoid bank conflicts without padding -- which lets the tile be
// filled by direct global->LDS loads (each wave instruction deposits 1 KB of consecutive LDS).
template <int D>
struct Tile {
    static constexpr int ROWB = D * 2;             // bytes per row
    static constexpr int BYTES = 64 * ROWB;
    static constexpr int CPR = D / 8;              // 16-byte chunks per row
    // XOR mask for the 16-byte chunk index of a row.  Rows r..r+15 must spread a fixed logical chunk over
    // all bank groups (ds_read_b128 fragments), while four consecutive rows must land in four different
    // 64-byte slots (the 4-row x 32-byte footprint of a ds_read_b64_tr_b16 lane block): both hold when the
    // row bits are rotated so that the low two select the slot and the next ones the chunk inside it.
    __device__ static __forceinline__ int swz(int row) {
        if (D == 128) { const int x = row & 15; return ((x & 3) << 2) | (x >> 2); }
        const int x = (row >> 1) & 7;
        return ((x & 1) << 2) | (x >> 1);
    }
};

__device__ __forceinline__ i32x4 make_rsrc_words(const void* base, uint32_t bytes) {
    const uint64_t p = (uint64_t)base;
    return i32x4{(int)(uint32_t)p, (int)(uint32_t)(p >> 32), (int)bytes, 0x00020000};
}
__device__ __forceinline__ void wait_dma() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// accumulator registers 8*half .. 8*half+7 -> bf16 operand
__device__ __forceinline__ bf16x8 pack8(const f32x16& a, int half) {
    union { uint32_t u[4]; bf16x8 v; } r;
#pragma unroll
    for (int i = 0; i < 4; i++) r.u[i] = pack_bf2(a[8 * half + 2 * i], a[8 * half + 2 * i + 1]);
    return r.v;
}

// Software-pipelined MFMA sequence: NGROUPS groups of G (fragment load, MFMA) pairs; the fragments of
// group g+1 are requested from LDS before the MFMAs of group g are issued, and a scheduling fence
// after every group keeps the compiler from re-serialising load -> wait -> MFMA.
template <int NGROUPS, int G, typename L, typename M>
__device__ __forceinline__ void mfma_pipeline(L load, M mma) {
    bf16x8 cur[G], nxt[G];
#pragma unroll
    for (int i = 0; i < G; i++) cur[i] = load(i);
#pragma unroll
    for (int g = 0; g < NGROUPS; g++) {
        if (g + 1 < NGROUPS) {
#pragma unroll
            for (int i = 0; i < G; i++) nxt[i] = load((g + 1) * G + i);
        }
#pragma unroll
        for (int i = 0; i < G; i++) mma(g * G + i, cur[i]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < G; i++) cur[i] = nxt[i];
    }
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

typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;

// LDS byte addresses of one lane's fragment reads of a staged tile; the tile's own address and the
// row-block / k-step displacements are compile-time constants that go into the instructions' offset fields.
template <int D>
struct FragAddr {
    uint32_t rows[D / 16], cols0[D / 32], cols1[D / 32];
    // rows: fragment of tile rows (lane%32), 8 channels 16kk + 8(lane/32) .. of k step kk
    // cols0/cols1: transposed fragment of channel block dt -- result row = tile column 32dt + (lane%32), the
    //   lane's 8 k values are tile rows 8j + 4(lane/32) + e (j = 0,1: cols0, cols1; e = 0..3) of a k step
    __device__ __forceinline__ void init(uint32_t base) {
        using TL = Tile<D>;
        const int l = threadIdx.x & 63;
        const int r = l & 31;
#pragma unroll
        for (int k = 0; k < D / 16; k++) rows[k] = base + r * TL::ROWB + (((2 * k + (l >> 5)) ^ TL::swz(r)) << 4);
        const int row = 4 * (l >> 5) + ((l & 15) >> 2);
#pragma unroll
        for (int t = 0; t < D / 32; t++) {
            const int col = 32 * t + 16 * ((l >> 4) & 1) + 4 * (l & 3);
            const int c = col >> 3, within = (col & 7) * 2;
            cols0[t] = base + row * TL::ROWB + ((c ^ TL::swz(row)) << 4) + within;
            cols1[t] = base + (row + 8) * TL::ROWB + ((c ^ TL::swz(row + 8)) << 4) + within;
        }
    }
    // the tables follow the tile to another LDS address
    __device__ __forceinline__ void shift(int by) {
#pragma unroll
        for (int k = 0; k < D / 16; k++) rows[k] += by;
#pragma unroll
        for (int t = 0; t < D / 32; t++) { cols0[t] += by; cols1[t] += by; }
    }
    __device__ __forceinline__ bf16x8 frag_rows(int disp, int rblk, int kk) const {
        return *(const lds_bf16x8*)(size_t)(rows[kk] + (uint32_t)(disp + rblk * 32 * Tile<D>::ROWB));
    }
    __device__ __forceinline__ bf16x8 frag_cols(int disp, int dt, int kk) const {
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(size_t)(cols0[dt] + (uint32_t)(disp + kk * 16 * Tile<D>::ROWB)));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(size_t)(cols1[dt] + (uint32_t)(disp + kk * 16 * Tile<D>::ROWB)));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
};

// Direct global->LDS loads of a tile, NW waves sharing it: instruction i of wave w deposits the 1 KB block
// w*PER_WAVE + i.  off[] is the lane part of its source byte offset (tile row and swizzled chunk, for rows of ld
// elements), computed once; the tile's own offset (first token, column) is a scalar added per instruction.  The
// whole offset goes through the buffer's range check, so rows past the buffer extent deposit zeros.
template <int D, int NW>
struct DmaLane {
    static constexpr int PER_WAVE = Tile<D>::BYTES / 1024 / NW;
    uint32_t off[PER_WAVE];
    __device__ __forceinline__ void init(int w, int ld) {
        const int L = threadIdx.x & 63;
#pragma unroll
        for (int i = 0; i < PER_WAVE; i++) {
            const int row = (w * PER_WAVE + i) * (1024 / Tile<D>::ROWB) + L / Tile<D>::CPR;
            const int logical = (L % Tile<D>::CPR) ^ Tile<D>::swz(row);
            off[i] = ((uint32_t)row * (uint32_t)ld + (uint32_t)(logical * 8)) * 2u;
            asm volatile("" : "+v"(off[i]));   // keep it in its register: cheaper than recomputing it at every use
        }
    }
    // lds_tile, w and base are wave-uniform
    __device__ __forceinline__ void issue(uint32_t lds_tile, i32x4 rs, int w, uint32_t base) const {
#pragma unroll
        for (int i = 0; i < PER_WAVE; i++) {
            const uint32_t dst = lds_tile + (uint32_t)(w * PER_WAVE + i) * 1024u;
            const uint32_t voff = off[i] + base;
            asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(dst), "v"(voff), "s"(rs) : "memory");
        }
    }
};

// Slots [I0, I1) of a stream of N MFMA slots: slot i requests the fragment of slot i + AHEAD from LDS, issues
// its MFMA and then the vector work `side(i)`, which the same wave issues while that MFMA occupies the matrix
// pipe; the fence after each slot keeps this order.  A call starts its own lookahead (slots I0 .. I0+AHEAD-1).
template <int I0, int I1, int N, int AHEAD, typename L, typename M, typename W>
__device__ __forceinline__ void mfma_stream(L load, M mma, W side) {
    bf16x8 f[N];
#pragma unroll
    for (int i = I0; i < I0 + AHEAD && i < I1; i++) f[i] = load(i);
#pragma unroll
    for (int i = I0; i < I1; i++) {
        if (i + AHEAD < I1) f[i + AHEAD] = load(i + AHEAD);
        mma(i, f[i]);
        side(i);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// ------------------------------------------------------------------ forward
// NPAR = 1: 4 waves, each 32 queries of the block's 128, walking the key tiles one by one.
// NPAR = 2: 8 waves; waves 4..7 repeat the queries of waves 0..3 and the two groups take the even and the odd
//   key tiles (two tiles per step), so the longest job of the launch -- the last query block -- is half as
//   long.  The two partial results (accumulator, running maximum, sum) are merged through LDS at the end,
//   always in the same order.
template <int D, int NPAR>
__global__ __launch_bounds__(ATHREADS * NPAR, NPAR == 1 ? 2 : 1) void k_attn_fwd(const bf16_t* __restrict__ qkv, int ld, uint32_t qkv_bytes,
                                                       bf16_t* __restrict__ o, float* __restrict__ lse, int S, int nh, int nkv, int B) {
    using TL = Tile<D>;
    constexpr int NW = 4 * NPAR;
    constexpr int STAGE = 2 * TL::BYTES;                              // K tile | V tile
    extern __shared__ __attribute__((aligned(1024))) char smem[];     // [wave group][stage][K|V]
    // flattened grid, last query block first: the long jobs of every head and sample are dispatched
    // before the short ones
    const int nhb = nh * B;
    const int qb = (int)(gridDim.x / nhb) - 1 - (int)(blockIdx.x / nhb), h = (blockIdx.x % nhb) % nh, b = (blockIdx.x % nhb) / nh;
    const int A = nh * D;
    const int kcol = A + (h / (nh / nkv)) * D;   // this query head's key head; its value head is nkv*D further
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, hf = lane >> 5;
    const int wq = wave & 3, par = wave >> 2;
    const int q0 = qb * 128 + wq * 32;
    const int query = q0 + (lane & 31);
    const uint32_t tokb = (uint32_t)b * S;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(qkv, qkv_bytes);
    const i32x4 rsw = make_rsrc_words(qkv, qkv_bytes);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem);
    DmaLane<D, NW> dl_;
    dl_.init(wave, ld);
    // step s brings key tiles NPAR*s .. NPAR*s + NPAR-1, tile p of them into wave group p's stage s&1
    auto issue = [&](int st, int s) {
#pragma unroll
        for (int p = 0; p < NPAR; p++) {
            const uint32_t row0 = (tokb + (uint32_t)(NPAR * s + p) * 64u) * (uint32_t)ld;
            const uint32_t dst = lds0 + (uint32_t)((2 * p + st) * STAGE);
            dl_.issue(dst, rsw, wave, (row0 + (uint32_t)kcol) * 2u);
            dl_.issue(dst + TL::BYTES, rsw, wave, (row0 + (uint32_t)(kcol + nkv * D)) * 2u);
        }
    };
    issue(0, 0);
    FragAddr<D> fa;
    fa.init(lds0 + (uint32_t)(par * 2 * STAGE));

    bf16x8 qf[D / 16];
    load_qfrag<D>(qf, rs, tokb + query, ld, h * D);

    f32x16 oacc[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) oacc[i][r] = 0.f;
    float m = -INFINITY, lsum = 0.f;
    const float c = LOG2E / sqrtf((float)D);
    // the register loads above are complete here, as far as the compiler's wait counters go: the loop must not
    // carry waits for them, because those would also wait for the tile loads in flight
#pragma unroll
    for (int kk = 0; kk < D / 16; kk++) asm volatile("" : "+v"(qf[kk]));

    const int q_last = min(qb * 128 + 127, S - 1);
    for (int s = 0; s * (64 * NPAR) <= q_last; s++) {
        wait_dma();
        __syncthreads();   // the tiles of step s are in LDS for everyone; everyone has finished with step s-1
        if ((s + 1) * (64 * NPAR) <= q_last) issue((s + 1) & 1, s + 1);
        const int kv0 = (NPAR * s + par) * 64;
        if (s) fa.shift((s & 1) ? STAGE : -STAGE);
        if (kv0 > q0 + 31) continue;  // every key of the tile lies after every query of this wave
        f32x16 sacc[2];
        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        // S^T = K Q^T: index -> (key half tl, k step kk); the first k step starts from a zero accumulator
        mfma_pipeline<2 * (D / 16) / 4, 4>(
            [&](int idx) { return fa.frag_rows(0, idx / (D / 16), idx % (D / 16)); },
            [&](int idx, bf16x8 f) {
                const int tl = idx / (D / 16), kk = idx % (D / 16);
                sacc[tl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, qf[kk], kk ? sacc[tl] : zero16, 0, 0, 0);
            });
        // raw scores; m and the exponent live in the log2 domain of the scaled scores: p = 2^(s*c - m)
        float tmax = -INFINITY;
        if (kv0 + 63 > q0) {   // tile touches the diagonal: drop keys after the query
#pragma unroll
            for (int tl = 0; tl < 2; tl++)
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int key = kv0 + 32 * tl + 8 * (r >> 2) + 4 * hf + (r & 3);
                    if (key > query) sacc[tl][r] = -INFINITY;
                }
        }
#pragma unroll
        for (int tl = 0; tl < 2; tl++)
#pragma unroll
            for (int r = 0; r < 16; r++) tmax = fmaxf(tmax, sacc[tl][r]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, WAVE)) * c;
        // The running reference m only moves when some query's tile maximum exceeds it by more than
        // 2^8: probabilities then stay below 256 (exact in fp32, representable in bf16) and the
        // rescale of the output accumulators is skipped for almost every tile.
        if (__any(tmax > m + 8.0f)) {
            const float mn = fmaxf(m, tmax);
            const float alpha = __builtin_amdgcn_exp2f(m - mn);
            lsum *= alpha;
            m = mn;
#pragma unroll
            for (int i = 0; i < D / 32; i++)
#pragma unroll
                for (int r = 0; r < 16; r++) oacc[i][r] *= alpha;
        }
        float psum = 0.f;
#pragma unroll
        for (int tl = 0; tl < 2; tl++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sacc[tl][r], c, -m));
                sacc[tl][r] = p;
                psum += p;
            }
        lsum += psum;
        bf16x8 pf[4];
#pragma unroll
        for (int kk = 0; kk < 4; kk++) pf[kk] = pack8(sacc[kk >> 1], kk & 1);
        // O^T += V^T P^T: index -> (key step kk, channel block dt)
        mfma_pipeline<4 * (D / 32) / 4, 4>(
            [&](int idx) { return fa.frag_cols(TL::BYTES, idx % (D / 32), idx / (D / 32)); },
            [&](int idx, bf16x8 f) {
                const int kk = idx / (D / 32), dt = idx % (D / 32);
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, pf[kk], oacc[dt], 0, 0, 0);
            });
    }
    if (NPAR == 2) {
        // merge the odd-tile group into the even-tile group: [query wave][register][lane] floats, then m and the sum
        __syncthreads();   // nobody reads a K/V tile any more and no DMA is in flight
        float* mo = reinterpret_cast<float*>(smem) + wq * ((D / 2 + 2) * WAVE);
        if (par == 1) {
#pragma unroll
            for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
                for (int r = 0; r < 16; r++) mo[(dt * 16 + r) * WAVE + lane] = oacc[dt][r];
            mo[(D / 2) * WAVE + lane] = m;
            mo[(D / 2 + 1) * WAVE + lane] = lsum;
        }
        __syncthreads();
        if (par == 1) return;
        const float m1 = mo[(D / 2) * WAVE + lane], l1 = mo[(D / 2 + 1) * WAVE + lane];
        const float mn = fmaxf(m, m1);
        const float a0 = __builtin_amdgcn_exp2f(m - mn), a1 = __builtin_amdgcn_exp2f(m1 - mn);   // a group without tiles has m = -inf, sum 0
#pragma unroll
        for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
            for (int r = 0; r < 16; r++) oacc[dt][r] = oacc[dt][r] * a0 + mo[(dt * 16 + r) * WAVE + lane] * a1;
        lsum = lsum * a0 + l1 * a1;
        m = mn;
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

// Backward of the rotary embedding on a gradient row held the accumulator way (block dt = channels 32dt .. +31,
// registers 4g+e = channels 8g + 4hf + e of the block): channel i of the first half pairs with i + D/2, which the
// same lane holds in block dt + D/64.  The pair is rotated by minus the angle of position `pos`
// (table: cos[rope_seq][D/2] then sin[rope_seq][D/2]), scaled by sc, rounded once and stored.
template <int D>
__device__ __forceinline__ void store_rope_bwd(bf16_t* row, const f32x16 (&acc)[D / 32], float sc, int hf, int pos,
                                                const float* __restrict__ rope, int rope_seq) {
    constexpr int HB = D / 64;
    const float* cs = rope + (size_t)pos * (D / 2);
    const float* sn = cs + (size_t)rope_seq * (D / 2);
#pragma unroll
    for (int dt = 0; dt < HB; dt++)
#pragma unroll
        for (int g = 0; g < 4; g++) {
            const int i = 32 * dt + 8 * g + 4 * hf;
            const float4 c4 = *reinterpret_cast<const float4*>(cs + i), s4 = *reinterpret_cast<const float4*>(sn + i);
            const float c[4] = {c4.x, c4.y, c4.z, c4.w}, sm[4] = {-s4.x, -s4.y, -s4.z, -s4.w};
            float oa[4], ob[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const float a = acc[dt][4 * g + e] * sc, b = acc[dt + HB][4 * g + e] * sc;
                oa[e] = a * c[e] - b * sm[e];
                ob[e] = b * c[e] + a * sm[e];
            }
            *reinterpret_cast<uint2*>(row + i) = make_uint2(pack_bf2(oa[0], oa[1]), pack_bf2(oa[2], oa[3]));
            *reinterpret_cast<uint2*>(row + i + D / 2) = make_uint2(pack_bf2(ob[0], ob[1]), pack_bf2(ob[2], ob[3]));
        }
}

// --------------------------------------------------------------- backward: dQ
// The job of query block qb of (head, sample) hb = h + nh*b.  NPAR as in k_attn_fwd: with 2, the even and the
// odd key tiles go to two groups of 4 waves whose dQ sums are added through LDS at the end.  Unless DELTA_GIVEN
// (dvec filled by k_attn_delta before), the job also forms delta = <dO, O> of its queries (each lane holds half a
// row of dO for the MFMAs anyway) and leaves it in dvec for the dK/dV kernel that follows.
// LDS: per wave group, two stages of (K tile | V tile).
template <int D, int NPAR, bool DELTA_GIVEN>
__device__ __forceinline__ void attn_bwd_dq_body(const int qb, const int hb, const bf16_t* __restrict__ qkv, int ld, uint32_t qkv_bytes,
                                                 const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout, uint32_t do_bytes,
                                                 const float* __restrict__ lse, float* __restrict__ dvec,
                                                 bf16_t* __restrict__ dqkv, int S, int nh, int nkv, int B,
                                                 const float* __restrict__ rope, int rope_seq) {
    using TL = Tile<D>;
    constexpr int NW = 4 * NPAR;
    constexpr int STAGE = 2 * TL::BYTES;                              // K tile | V tile
    extern __shared__ __attribute__((aligned(1024))) char smem[];     // [wave group][stage][K|V]
    const int h = hb % nh, b = hb / nh;
    const int A = nh * D;
    const int kcol = A + (h / (nh / nkv)) * D;   // this query head's key head; its value head is nkv*D further
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, hf = lane >> 5;
    const int wq = wave & 3, par = wave >> 2;
    const int q0 = qb * 128 + wq * 32;
    const int query = q0 + (lane & 31);
    const uint32_t tokb = (uint32_t)b * S;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(qkv, qkv_bytes);
    const __amdgpu_buffer_rsrc_t rsdo = make_rsrc(dout, do_bytes);
    const i32x4 rsw = make_rsrc_words(qkv, qkv_bytes);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem);
    DmaLane<D, NW> dl_;
    dl_.init(wave, ld);
    // step s brings key tiles NPAR*s .. NPAR*s + NPAR-1, tile p of them into wave group p's stage s&1
    auto issue = [&](int st, int s) {
#pragma unroll
        for (int p = 0; p < NPAR; p++) {
            const uint32_t row0 = (tokb + (uint32_t)(NPAR * s + p) * 64u) * (uint32_t)ld;
            const uint32_t dst = lds0 + (uint32_t)((2 * p + st) * STAGE);
            dl_.issue(dst, rsw, wave, (row0 + (uint32_t)kcol) * 2u);
            dl_.issue(dst + TL::BYTES, rsw, wave, (row0 + (uint32_t)(kcol + nkv * D)) * 2u);
        }
    };
    issue(0, 0);
    FragAddr<D> fa;
    fa.init(lds0 + (uint32_t)(par * 2 * STAGE));

    bf16x8 qf[D / 16], dof[D / 16];
    load_qfrag<D>(qf, rs, tokb + query, ld, h * D);
    load_qfrag<D>(dof, rsdo, tokb + query, A, h * D);
    const float sc = 1.0f / sqrtf((float)D);
    const float c = LOG2E * sc;
    // delta: this lane's half of the row, plus the other half from lane ^ 32 (or, when a kernel before this one
    // has left it in dvec, read from there)
    float dl = 0.f;
    if (!DELTA_GIVEN) {
        const __amdgpu_buffer_rsrc_t rso = make_rsrc(o, do_bytes);
        bf16x8 of[D / 16];
        load_qfrag<D>(of, rso, tokb + query, A, h * D);
#pragma unroll
        for (int kk = 0; kk < D / 16; kk++)
#pragma unroll
            for (int e = 0; e < 8; e++) dl = fmaf((float)dof[kk][e], (float)of[kk][e], dl);
        dl += __shfl_xor(dl, 32, WAVE);
    }
    float L = 0.f;
    if (query < S) {
        const size_t at = ((size_t)b * nh + h) * S + query;
        L = lse[at] * LOG2E;
        if (DELTA_GIVEN) dl = dvec[at];
        else if (par == 0 && hf == 0) dvec[at] = dl;
    }
    // every register load above is complete here, as far as the compiler's wait counters go: the loop must not
    // carry waits for them, because those would also wait for the tile loads in flight
#pragma unroll
    for (int kk = 0; kk < D / 16; kk++) asm volatile("" : "+v"(qf[kk]), "+v"(dof[kk]));
    asm volatile("" : "+v"(L), "+v"(dl));
    f32x16 dq[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) dq[i][r] = 0.f;
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // One key tile (64 keys) against this wave's 32 queries.  MFMA slots, K = D/16 k steps:
    //   [0, 2K)   S^T and dP^T of keys 0..31   (K Q^T, V dO^T; k step i/2, alternating)
    //   [2K, 4K)  the same for keys 32..63, with the softmax-gradient arithmetic of keys 0..31 in the shadow
    //   then      dQ^T += K^T dS^T over key steps 0,1 (keys 0..31), with the arithmetic of keys 32..63 in the
    //             shadow, and over key steps 2,3.
    // On a tile that touches the diagonal, the entries of keys after the query are cleared in the packed dS^T.
    const int q_last = min(qb * 128 + 127, S - 1);
    for (int s = 0; s * (64 * NPAR) <= q_last; s++) {
        wait_dma();
        __syncthreads();   // the tiles of step s are in LDS for everyone; everyone has finished with step s-1
        if ((s + 1) * (64 * NPAR) <= q_last) issue((s + 1) & 1, s + 1);
        const int kv0 = (NPAR * s + par) * 64;
        if (s) fa.shift((s & 1) ? STAGE : -STAGE);
        if (kv0 > q0 + 31) continue;
        const bool diag = kv0 + 63 > q0;
        constexpr int K2 = 2 * (D / 16), NQ = 4 * (D / 32);
        f32x16 sacc[2], pacc[2];
        union { uint32_t u[4]; bf16x8 v; } sf[4];
        const int qrel = query - kv0 - 4 * hf;      // a register's key offset inside the tile (without its lane part) that equals the query
        auto grad = [&](int tl, int r) {            // element r of key half tl: p, then dS^T (before the 1/sqrt(d) factor)
            const float p = __builtin_amdgcn_exp2f(fmaf(sacc[tl][r], c, -L));
            sacc[tl][r] = p * (pacc[tl][r] - dl);
            if (r & 1) sf[2 * tl + (r >> 3)].u[(r & 7) >> 1] = pack_bf2(sacc[tl][r - 1], sacc[tl][r]);
        };
        auto clear_future = [&](int tl, int r0) {   // packed pairs (r-1, r), r0 <= r < r0+8, of key half tl: drop keys after the query
            asm volatile("" ::: "memory");          // a real branch around the rare case, not selects on every tile
#pragma unroll
            for (int r = r0 + 1; r < r0 + 8; r += 2) {
                const int k1 = 32 * tl + 8 * (r >> 2) + (r & 3);    // key offset of element r; element r-1 is the key before it
                uint32_t& w = sf[2 * tl + (r >> 3)].u[(r & 7) >> 1];
                w = k1 <= qrel ? w : (k1 - 1 <= qrel ? (w & 0xFFFFu) : 0u);
            }
        };
        auto load = [&](int i) {
            if (i < 2 * K2) return fa.frag_rows((i & 1) ? TL::BYTES : 0, i / K2, (i % K2) >> 1);
            const int j = i - 2 * K2;
            return fa.frag_cols(0, j % (D / 32), j / (D / 32));
        };
        auto mma = [&](int i, bf16x8 f) {
            if (i < 2 * K2) {
                const int tl = i / K2, kk = (i % K2) >> 1;
                if (i & 1) pacc[tl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, dof[kk], kk ? pacc[tl] : zero16, 0, 0, 0);
                else sacc[tl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, qf[kk], kk ? sacc[tl] : zero16, 0, 0, 0);
            } else {
                const int j = i - 2 * K2, kk = j / (D / 32), dt = j % (D / 32);
                dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, sf[kk].v, dq[dt], 0, 0, 0);
            }
        };
        // slots [0, 2K2): S^T, dP^T of both halves; the arithmetic of half 0 rides on the second K2 slots
        constexpr int PER0 = (16 + K2 - 1) / K2;
        mfma_stream<0, 2 * K2, 2 * K2 + NQ, 2>(load, mma, [&](int i) {
            if (i >= K2) {
#pragma unroll
                for (int e = 0; e < PER0; e++) { const int r = (i - K2) * PER0 + e; if (r < 16) grad(0, r); }
            }
        });
        if (diag) { clear_future(0, 0); clear_future(0, 8); }
        // slots of dQ^T: key steps 0,1 with the first half of the arithmetic of key half 1 (8 elements), key step 2
        // with the second, key step 3
        constexpr int DT = D / 32;
        constexpr int PERA = (8 + 2 * DT - 1) / (2 * DT), PERB = (8 + DT - 1) / DT;
        mfma_stream<2 * K2, 2 * K2 + 2 * DT, 2 * K2 + NQ, 2>(load, mma, [&](int i) {
#pragma unroll
            for (int e = 0; e < PERA; e++) { const int r = (i - 2 * K2) * PERA + e; if (r < 8) grad(1, r); }
        });
        if (diag) clear_future(1, 0);
        mfma_stream<2 * K2 + 2 * DT, 2 * K2 + 3 * DT, 2 * K2 + NQ, 2>(load, mma, [&](int i) {
#pragma unroll
            for (int e = 0; e < PERB; e++) { const int r = 8 + (i - 2 * K2 - 2 * DT) * PERB + e; if (r < 16) grad(1, r); }
        });
        if (diag) clear_future(1, 8);
        mfma_stream<2 * K2 + 3 * DT, 2 * K2 + NQ, 2 * K2 + NQ, 2>(load, mma, [&](int) {});
    }
    if (NPAR == 2) {
        __syncthreads();   // nobody reads a K/V tile any more and no DMA is in flight
        float* mo = reinterpret_cast<float*>(smem) + wq * ((D / 2) * WAVE);
        if (par == 1) {
#pragma unroll
            for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
                for (int r = 0; r < 16; r++) mo[(dt * 16 + r) * WAVE + lane] = dq[dt][r];
        }
        __syncthreads();
        if (par == 1) return;
#pragma unroll
        for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
            for (int r = 0; r < 16; r++) dq[dt][r] += mo[(dt * 16 + r) * WAVE + lane];
    }
    if (query < S) {
        bf16_t* row = dqkv + (size_t)(tokb + query) * ld + h * D;
        if (rope) {
            store_rope_bwd<D>(row, dq, sc, hf, query, rope, rope_seq);
            return;
        }
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
// The job of key block kb; rem = (sample, key/value head, slice of its query heads).  8 waves: wave = (query
// half qh, key group kw).  The workgroup owns 128 keys (4 groups of 32) and walks the query tiles from its
// diagonal to the end; of every 64-query tile a wave takes the 32 queries of its half.  The two halves' dK, dV
// sums are added through LDS at the end (fixed order: deterministic).
constexpr int KVTHREADS = 512;
template <int D>
__device__ __forceinline__ void attn_bwd_dkv_body(const int kb, const int rem, const bf16_t* __restrict__ qkv, int ld, uint32_t qkv_bytes,
                                                  const bf16_t* __restrict__ dout, uint32_t do_bytes,
                                                  const float* __restrict__ lse, const float* __restrict__ dvec,
                                                  bf16_t* __restrict__ dqkv, int S, int nh, int nkv, int B,
                                                  int hs, float* __restrict__ part, const float* __restrict__ rope, int rope_seq) {
    using TL = Tile<D>;
    constexpr int NW = KVTHREADS / WAVE;
    constexpr int STAGE = 2 * TL::BYTES;                              // Q tile | dO tile
    // LDS: two Q|dO stages, the workgroup's K (2 tiles) and V (2 tiles), then lse/delta[2][64|64]
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const char* sKV = smem + 2 * STAGE;
    float* sLD = reinterpret_cast<float*>(smem + 2 * STAGE + 4 * TL::BYTES);
    // flattened grid over (key block, sample, key/value head, slice of its query heads): key block first (block 0
    // has the most query tiles), so the long jobs of every head and sample are dispatched before the short ones
    const int b = rem / (nkv * hs), hk = (rem % (nkv * hs)) / hs, ps = rem % hs;
    // the key/value head collects the gradients of query heads hk*(nh/nkv) .. ; this workgroup sums G of them
    // (slice ps of hs) and, when hs > 1, leaves fp32 partial sums in part[ps][dK|dV][token][nkv*D]
    const int A = nh * D, G = nh / nkv / hs, h_first = hk * (nh / nkv) + ps * G;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5;
    const int kw = wave & 3, qh = wave >> 2;
    const int k0 = kb * 128 + kw * 32;
    const int key = k0 + (lane & 31);
    const uint32_t tokb = (uint32_t)b * S;
    const i32x4 rsw = make_rsrc_words(qkv, qkv_bytes);
    const i32x4 rswdo = make_rsrc_words(dout, do_bytes);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    DmaLane<D, NW> lane_q, lane_o;            // rows of ld elements (q | k | v) and of A elements (dO)
    lane_q.init(wave_s, ld);
    lane_o.init(wave_s, A);
    // work items: for each of the G query heads, the query tiles from the key block's diagonal to the end;
    // an item is (query head h, step s) with its 64 queries starting at kb*128 + 64*s
    const int nsteps = (S - kb * 128 + 63) / 64, nitems = G * nsteps;
    auto issue = [&](int st, int h, int sq) {
        const uint32_t row0 = tokb + (uint32_t)(kb * 128 + sq * 64);
        lane_q.issue(lds0 + st * STAGE, rsw, wave_s, (row0 * (uint32_t)ld + (uint32_t)(h * D)) * 2u);
        lane_o.issue(lds0 + st * STAGE + TL::BYTES, rswdo, wave_s, (row0 * (uint32_t)A + (uint32_t)(h * D)) * 2u);
    };
    // lse (log2 domain) and delta of the 64 queries of an item: thread i < 64 -> lse, 64 <= i < 128 -> delta
    auto stat = [&](int h, int sq) -> float {
        const int i = threadIdx.x & 63, qq = kb * 128 + sq * 64 + i;
        if (threadIdx.x >= 128 || qq >= S) return 0.f;
        const size_t at = ((size_t)b * nh + h) * S + qq;
        return threadIdx.x < 64 ? lse[at] * LOG2E : dvec[at];
    };
    // K, V of keys kb*128 .. +127: resident for the whole kernel (first wait_dma below covers them)
#pragma unroll
    for (int i = 0; i < 2; i++) {
        const uint32_t row0 = (tokb + (uint32_t)(kb * 128 + 64 * i)) * (uint32_t)ld;
        lane_q.issue(lds0 + 2 * STAGE + i * TL::BYTES, rsw, wave_s, (row0 + (uint32_t)(A + hk * D)) * 2u);
        lane_q.issue(lds0 + 2 * STAGE + (2 + i) * TL::BYTES, rsw, wave_s, (row0 + (uint32_t)(A + (nkv + hk) * D)) * 2u);
    }
    issue(0, h_first, 0);
    float nstat = stat(h_first, 0);
    int cs = 0;                                            // step of the item being worked on
    int ih = nsteps > 1 ? h_first : h_first + 1, is = nsteps > 1 ? 1 : 0;   // the item after it
    // fragment addresses: fq of the stage tiles (Q at +0, dO at +BYTES; moved to the other stage after every
    // item), fk of this wave's 32 keys in the resident K tile (V at +2*BYTES)
    FragAddr<D> fq, fk;
    fq.init(lds0 + (uint32_t)(qh * 32 * TL::ROWB));   // this wave's 32 queries of a tile: row block qh = key steps 2qh, 2qh+1
    fk.init(lds0 + (uint32_t)(2 * STAGE + (kw >> 1) * TL::BYTES + (kw & 1) * 32 * TL::ROWB));
    const float sc = 1.0f / sqrtf((float)D);
    const float c = LOG2E * sc;
    f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) { dk[i][r] = 0.f; dv[i][r] = 0.f; }

    for (int t = 0; t < nitems; t++, cs = is, ih += (is + 1 == nsteps), is = (is + 1 == nsteps) ? 0 : is + 1) {
        const int qt = kb * 128 + cs * 64;
        if (threadIdx.x < 128) sLD[(t & 1) * 128 + threadIdx.x] = nstat;   // lse / delta of item t (fetched a step ago)
        wait_dma();
        __syncthreads();   // item t and its lse/delta are in LDS for everyone; everyone has finished with item t-1
        if (t + 1 < nitems) { issue((t + 1) & 1, ih, is); nstat = stat(ih, is); }
        if (t) fq.shift((t & 1) ? STAGE : -STAGE);
        const float* sL = sLD + (t & 1) * 128;
        const float* sD = sL + 64;
        const int q0 = qt + 32 * qh;                 // this wave's 32 queries of the tile
        if (q0 + 31 < k0) continue;                  // all of them precede every key of this wave
        f32x16 sacc, pacc;
        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        // S = Q K^T and dP = dO V^T.  Fragment stream: per k step kk the four fragments Q, K, dO, V;
        // an MFMA is issued when its second operand arrives (odd index).
        {
            bf16x8 first;
            mfma_pipeline<4 * (D / 16) / 4, 4>(
                [&](int idx) {
                    const int kk = idx >> 2, w = idx & 3;
                    return w == 0 ? fq.frag_rows(0, 0, kk) : w == 1 ? fk.frag_rows(0, 0, kk)
                         : w == 2 ? fq.frag_rows(TL::BYTES, 0, kk) : fk.frag_rows(2 * TL::BYTES, 0, kk);
                },
                [&](int idx, bf16x8 f) {
                    const int w = idx & 3, kk = idx >> 2;
                    if (w == 0 || w == 2) first = f;
                    else if (w == 1) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(first, f, kk ? sacc : zero16, 0, 0, 0);
                    else pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(first, f, kk ? pacc : zero16, 0, 0, 0);
                });
        }
        union { uint32_t u[4]; bf16x8 v; } pf[2], sf[2];
#pragma unroll
        for (int g = 0; g < 4; g++) {
            const int qi = 32 * qh + 8 * g + 4 * hf;
            const float4 l4 = *reinterpret_cast<const float4*>(&sL[qi]);
            const float4 d4 = *reinterpret_cast<const float4*>(&sD[qi]);
            const float ls[4] = {l4.x, l4.y, l4.z, l4.w}, ds[4] = {d4.x, d4.y, d4.z, d4.w};
            float pv[4], sv[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                pv[e] = __builtin_amdgcn_exp2f(fmaf(sacc[4 * g + e], c, -ls[e]));
                sv[e] = pv[e] * (pacc[4 * g + e] - ds[e]);
            }
            pf[g >> 1].u[2 * (g & 1)] = pack_bf2(pv[0], pv[1]);
            pf[g >> 1].u[2 * (g & 1) + 1] = pack_bf2(pv[2], pv[3]);
            sf[g >> 1].u[2 * (g & 1)] = pack_bf2(sv[0], sv[1]);
            sf[g >> 1].u[2 * (g & 1) + 1] = pack_bf2(sv[2], sv[3]);
        }
        if ((q0 < k0 + 31) || (q0 + 31 >= S)) {
            // the tile touches the diagonal or the end of the sequence: clear the entries whose query precedes the
            // key or does not exist (a real branch around the rare case, not selects on every tile)
            asm volatile("" ::: "memory");
#pragma unroll
            for (int w = 0; w < 8; w++) {
                const int q = q0 + 8 * (w >> 1) + 4 * hf + 2 * (w & 1);   // query of the pair's first element
                const uint32_t keep = (key <= q && q < S ? 0xFFFFu : 0u) | (key <= q + 1 && q + 1 < S ? 0xFFFF0000u : 0u);
                pf[w >> 2].u[w & 3] &= keep;
                sf[w >> 2].u[w & 3] &= keep;
            }
        }
        // dV^T += dO^T P and dK^T += Q^T dS over this wave's 32 queries (k steps 2qh, 2qh+1 of the tile):
        // index -> (query step, channel block dt, {dO, Q})
        mfma_pipeline<2 * (D / 32) * 2 / 4, 4>(
            [&](int idx) { return fq.frag_cols((idx & 1) ? 0 : TL::BYTES, (idx >> 1) % (D / 32), (idx >> 1) / (D / 32)); },
            [&](int idx, bf16x8 f) {
                const int dt = (idx >> 1) % (D / 32), kk = (idx >> 1) / (D / 32);
                if (idx & 1) dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, sf[kk].v, dk[dt], 0, 0, 0);
                else dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, pf[kk].v, dv[dt], 0, 0, 0);
            });
    }
    // add the second query half's sums to the first's: [kw][register][lane] floats in the stage memory
    float* red = reinterpret_cast<float*>(smem);
    constexpr int R = (D / 32) * 16;
    __syncthreads();
    if (qh == 1) {
#pragma unroll
        for (int i = 0; i < D / 32; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) red[(kw * R + i * 16 + r) * 64 + lane] = dk[i][r];
    }
    __syncthreads();
    if (qh == 0) {
#pragma unroll
        for (int i = 0; i < D / 32; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) dk[i][r] += red[(kw * R + i * 16 + r) * 64 + lane];
    }
    __syncthreads();
    if (qh == 1) {
#pragma unroll
        for (int i = 0; i < D / 32; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) red[(kw * R + i * 16 + r) * 64 + lane] = dv[i][r];
    }
    __syncthreads();
    if (hs > 1) {
        // Partial sums leave through a wave-private LDS patch in the K/V area (no longer read by anyone): a lane
        // holds 4-channel pieces of one key row, the patch hands back whole rows, 16 bytes a lane.
        if (qh != 0) return;
        constexpr int CH = D / 4, RP = WAVE / CH;             // 16-byte chunks per row, rows per store instruction
        char* const patch = smem + 2 * STAGE + kw * (32 * D * 4);
        const int Akv = nkv * D;
        const size_t plane = (size_t)B * S * Akv;
#pragma unroll
        for (int which = 0; which < 2; which++) {
            const int r_w = lane & 31;
#pragma unroll
            for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    float4 v;
                    if (which == 0) {
                        v = make_float4(dk[dt][4 * g] * sc, dk[dt][4 * g + 1] * sc, dk[dt][4 * g + 2] * sc, dk[dt][4 * g + 3] * sc);
                    } else {
                        const float* rp = &red[(kw * R + dt * 16 + 4 * g) * 64 + lane];
                        v = make_float4(dv[dt][4 * g] + rp[0], dv[dt][4 * g + 1] + rp[64], dv[dt][4 * g + 2] + rp[128], dv[dt][4 * g + 3] + rp[192]);
                    }
                    const int chunk = 8 * dt + 2 * g + hf;
                    *reinterpret_cast<float4*>(patch + r_w * (D * 4) + ((chunk ^ (r_w & (CH - 1))) << 4)) = v;
                }
            float* const dst = part + (size_t)(ps * 2 + which) * plane + (size_t)hk * D;
#pragma unroll
            for (int rr = 0; rr < 32; rr += RP) {
                const int row = rr + lane / CH, chunk = lane % CH;
                const float4 v = *reinterpret_cast<const float4*>(patch + row * (D * 4) + ((chunk ^ (row & (CH - 1))) << 4));
                if (k0 + row < S) *reinterpret_cast<float4*>(dst + (size_t)(tokb + k0 + row) * Akv + 4 * chunk) = v;
            }
        }
        return;
    }
    if (qh == 0 && key < S) {
        bf16_t* krow = dqkv + (size_t)(tokb + key) * ld + A + hk * D;
        bf16_t* vrow = krow + nkv * D;
#pragma unroll
        for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                float w[4];
#pragma unroll
                for (int e = 0; e < 4; e++) w[e] = dv[dt][4 * g + e] + red[(kw * R + dt * 16 + 4 * g + e) * 64 + lane];
                uint2 v;
                if (!rope) {
                    v.x = pack_bf2(dk[dt][4 * g] * sc, dk[dt][4 * g + 1] * sc);
                    v.y = pack_bf2(dk[dt][4 * g + 2] * sc, dk[dt][4 * g + 3] * sc);
                    *reinterpret_cast<uint2*>(krow + 32 * dt + 8 * g + 4 * hf) = v;
                }
                v.x = pack_bf2(w[0], w[1]);
                v.y = pack_bf2(w[2], w[3]);
                *reinterpret_cast<uint2*>(vrow + 32 * dt + 8 * g + 4 * hf) = v;
            }
        if (rope) store_rope_bwd<D>(krow, dk, sc, hf, key, rope, rope_seq);
    }
}

// flattened grid, last query block first (see k_attn_fwd)
template <int D, int NPAR>
__global__ __launch_bounds__(ATHREADS * NPAR, NPAR == 1 ? 2 : 1) void k_attn_bwd_dq(const bf16_t* __restrict__ qkv, int ld, uint32_t qkv_bytes,
                                                          const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout, uint32_t do_bytes,
                                                          const float* __restrict__ lse, float* __restrict__ dvec,
                                                          bf16_t* __restrict__ dqkv, int S, int nh, int nkv, int B,
                                                          const float* __restrict__ rope, int rope_seq) {
    const int nhb = nh * B;
    attn_bwd_dq_body<D, NPAR, false>((int)(gridDim.x / nhb) - 1 - (int)(blockIdx.x / nhb), blockIdx.x % nhb, qkv, ld, qkv_bytes, o, dout, do_bytes,
                                     lse, dvec, dqkv, S, nh, nkv, B, rope, rope_seq);
}

// flattened grid over (key block, sample, key/value head, slice of its query heads): key block first (block 0
// has the most query tiles), so the long jobs of every head and sample are dispatched before the short ones
template <int D>
__global__ __launch_bounds__(KVTHREADS) void k_attn_bwd_dkv(const bf16_t* __restrict__ qkv, int ld, uint32_t qkv_bytes,
                                                            const bf16_t* __restrict__ dout, uint32_t do_bytes,
                                                            const float* __restrict__ lse, const float* __restrict__ dvec,
                                                            bf16_t* __restrict__ dqkv, int S, int nh, int nkv, int B,
                                                            int hs, float* __restrict__ part, const float* __restrict__ rope, int rope_seq) {
    const int nkb = nkv * hs * B;
    attn_bwd_dkv_body<D>(blockIdx.x / nkb, blockIdx.x % nkb, qkv, ld, qkv_bytes, dout, do_bytes, lse, dvec, dqkv, S, nh, nkv, B, hs, part,
                         rope, rope_seq);
}

// Both backward passes in one launch, for launches so small that each pass alone is bound by its longest job (the
// last query block, the first key block) while most CUs idle: the jobs of the two passes are dealt out together,
// longest first -- level l holds the dK/dV jobs of key block l and then the dQ jobs of query block n-1-l -- so the
// short jobs of one pass fill the CUs that the other leaves.  delta comes from k_attn_delta, launched before.
template <int D>
__global__ __launch_bounds__(KVTHREADS) void k_attn_bwd_both(const bf16_t* __restrict__ qkv, int ld, uint32_t qkv_bytes,
                                                             const bf16_t* __restrict__ dout, uint32_t do_bytes,
                                                             const float* __restrict__ lse, float* __restrict__ dvec,
                                                             bf16_t* __restrict__ dqkv, int S, int nh, int nkv, int B,
                                                             int hs, float* __restrict__ part, const float* __restrict__ rope, int rope_seq) {
    const int nkvj = nkv * hs * B, nqj = nh * B, per = nkvj + nqj;
    const int level = blockIdx.x / per, nblk = gridDim.x / per;
    const int r = blockIdx.x % per;
    if (r < nkvj) attn_bwd_dkv_body<D>(level, r, qkv, ld, qkv_bytes, dout, do_bytes, lse, dvec, dqkv, S, nh, nkv, B, hs, part, rope, rope_seq);
    else attn_bwd_dq_body<D, 2, true>(nblk - 1 - level, r - nkvj, qkv, ld, qkv_bytes, nullptr, dout, do_bytes, lse, dvec, dqkv, S, nh, nkv, B,
                                      rope, rope_seq);
}

// delta[b, h, s] = <dO[s, h, :], O[s, h, :]>.  Two threads per (token, head): thread hf takes the 8-channel groups
// 16kk + 8hf .. of the row, in the order and with the arithmetic of the dQ kernel's own delta.
template <int D>
__global__ __launch_bounds__(256) void k_attn_delta(const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout, float* __restrict__ dvec,
                                                    int S, int nh, long rows) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long row = i >> 1;                    // token * nh + head
    const int hf = (int)(i & 1);
    float dl = 0.f;
    if (row < rows) {
        const bf16_t* po = o + row * D + 8 * hf;
        const bf16_t* pd = dout + row * D + 8 * hf;
#pragma unroll
        for (int kk = 0; kk < D / 16; kk++) {
            const uint4 a = *reinterpret_cast<const uint4*>(pd + 16 * kk), c = *reinterpret_cast<const uint4*>(po + 16 * kk);
            const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, cw[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
            for (int e = 0; e < 4; e++) {
                dl = fmaf(lo_bf(aw[e]), lo_bf(cw[e]), dl);
                dl = fmaf(hi_bf(aw[e]), hi_bf(cw[e]), dl);
            }
        }
    }
    dl += __shfl_xor(dl, 1, WAVE);
    if (row < rows && hf == 0) {
        const long tok = row / nh;
        const int h = (int)(row % nh);
        dvec[((tok / S) * nh + h) * S + tok % S] = dl;
    }
}

// Sums the hs partial dK and dV planes of grouped heads in a fixed order and writes them, rounded to bf16,
// into the k and v columns of dqkv.  A thread owns 4 consecutive channels c.. of the first half of one key/value
// head of one token together with their partners c + D/2, so that it can also take the rotary embedding back
// out of dK (rope != null: rotation by minus the token's angle; table as in store_rope_bwd).
__global__ __launch_bounds__(256) void k_attn_dkv_reduce(const float* __restrict__ part, int hs, long tokens, int Akv, int D, int S,
                                                         bf16_t* __restrict__ dqkv, int ld, int A,
                                                         const float* __restrict__ rope, int rope_seq) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int per_tok = Akv / 8, half = D / 2;
    if (i >= tokens * per_tok) return;
    const long tok = i / per_tok;
    const int j = (int)(i % per_tok);
    const int c = (j % (half / 4)) * 4;                     // channel inside the head's first half
    const int col = (j / (half / 4)) * D + c;
    const size_t plane = (size_t)tokens * Akv;
    const float* p = part + (size_t)tok * Akv + col;
    float4 k0 = *reinterpret_cast<const float4*>(p), k1 = *reinterpret_cast<const float4*>(p + half);
    float4 v0 = *reinterpret_cast<const float4*>(p + plane), v1 = *reinterpret_cast<const float4*>(p + plane + half);
    for (int s = 1; s < hs; s++) {
        const float* q = p + (size_t)(2 * s) * plane;
        const float4 a0 = *reinterpret_cast<const float4*>(q), a1 = *reinterpret_cast<const float4*>(q + half);
        const float4 b0 = *reinterpret_cast<const float4*>(q + plane), b1 = *reinterpret_cast<const float4*>(q + plane + half);
        k0.x += a0.x; k0.y += a0.y; k0.z += a0.z; k0.w += a0.w;
        k1.x += a1.x; k1.y += a1.y; k1.z += a1.z; k1.w += a1.w;
        v0.x += b0.x; v0.y += b0.y; v0.z += b0.z; v0.w += b0.w;
        v1.x += b1.x; v1.y += b1.y; v1.z += b1.z; v1.w += b1.w;
    }
    if (rope) {
        const float* cs = rope + (size_t)(tok % S) * half + c;
        const float* sn = cs + (size_t)rope_seq * half;
        const float4 c4 = *reinterpret_cast<const float4*>(cs), s4 = *reinterpret_cast<const float4*>(sn);
        const float cc[4] = {c4.x, c4.y, c4.z, c4.w}, sm[4] = {-s4.x, -s4.y, -s4.z, -s4.w};
        const float a[4] = {k0.x, k0.y, k0.z, k0.w}, b[4] = {k1.x, k1.y, k1.z, k1.w};
        float oa[4], ob[4];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            oa[e] = a[e] * cc[e] - b[e] * sm[e];
            ob[e] = b[e] * cc[e] + a[e] * sm[e];
        }
        k0 = make_float4(oa[0], oa[1], oa[2], oa[3]);
        k1 = make_float4(ob[0], ob[1], ob[2], ob[3]);
    }
    bf16_t* row = dqkv + (size_t)tok * ld + A + col;
    *reinterpret_cast<uint2*>(row) = make_uint2(pack_bf2(k0.x, k0.y), pack_bf2(k0.z, k0.w));
    *reinterpret_cast<uint2*>(row + half) = make_uint2(pack_bf2(k1.x, k1.y), pack_bf2(k1.z, k1.w));
    *reinterpret_cast<uint2*>(row + Akv) = make_uint2(pack_bf2(v0.x, v0.y), pack_bf2(v0.z, v0.w));
    *reinterpret_cast<uint2*>(row + Akv + half) = make_uint2(pack_bf2(v1.x, v1.y), pack_bf2(v1.z, v1.w));
}

// ---------------------------------------------------------------- launchers
// Into how many slices the query heads of a key/value head are cut for dK, dV: one (the workgroup of a key block sums
// all of them in registers) unless that leaves too few workgroups to balance the causal triangle over the chip.
static int dkv_head_slices(int B, int S, int nh, int nkv) {
    const int G = nh / nkv;
    const long wgs = (long)((S + 127) / 128) * nkv * B;
    int hs = 1;
    while (hs < G && wgs * hs < 4 * 256) {
        do ++hs; while (G % hs);
    }
    return hs;
}

size_t attn_bf16_bwd_scratch_bytes(int B, int S, int nh, int nkv, int d) {
    const int hs = dkv_head_slices(B, S, nh, nkv);
    return hs > 1 ? (size_t)hs * 2 * B * S * nkv * d * sizeof(float) : 0;
}

template <typename K>
static hipError_t set_lds(K kern, int bytes) {
    return bytes > 48 * 1024 ? hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) : hipSuccess;
}

// Key tiles are split between two wave groups (NPAR = 2) when the launch is bound by its longest job: few enough
// workgroups that all of them run at once, i.e. no later jobs to fill the CUs that the short ones leave.
static bool split_keys(unsigned grid, int S) { return S >= 1024 && grid <= 2 * 256; }

template <int D>
static hipError_t fwd_d(const void* qkv, int ld, uint32_t bytes, void* o, float* lse, int B, int S, int nh, int nkv, hipStream_t st) {
    const unsigned grid = (unsigned)((S + 127) / 128) * nh * B;
    if (split_keys(grid, S)) {
        constexpr int LDS = 8 * Tile<D>::BYTES;
        hipError_t e = set_lds(k_attn_fwd<D, 2>, LDS);
        if (e != hipSuccess) return e;
        k_attn_fwd<D, 2><<<grid, 2 * ATHREADS, LDS, st>>>((const bf16_t*)qkv, ld, bytes, (bf16_t*)o, lse, S, nh, nkv, B);
    } else {
        constexpr int LDS = 4 * Tile<D>::BYTES;
        hipError_t e = set_lds(k_attn_fwd<D, 1>, LDS);
        if (e != hipSuccess) return e;
        k_attn_fwd<D, 1><<<grid, ATHREADS, LDS, st>>>((const bf16_t*)qkv, ld, bytes, (bf16_t*)o, lse, S, nh, nkv, B);
    }
    return hipGetLastError();
}

template <int D>
static hipError_t bwd_d(const void* qkv, int ld, uint32_t bytes, const void* o, const void* dout, uint32_t do_bytes,
                        const float* lse, float* dvec, void* dqkv, float* scratch, int B, int S, int nh, int nkv,
                        const float* rope, int rope_seq, hipStream_t st) {
    constexpr int LDS_KV = 8 * Tile<D>::BYTES + 1024;
    hipError_t e = set_lds(k_attn_bwd_dkv<D>, LDS_KV);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)((S + 127) / 128) * nh * B;
    const int hs = dkv_head_slices(B, S, nh, nkv);
    if (hs > 1 && !scratch) return hipErrorInvalidValue;
    const unsigned grid_kv = (unsigned)((S + 127) / 128) * nkv * hs * B;
    if (split_keys(grid, S)) {
        e = set_lds(k_attn_bwd_both<D>, LDS_KV);
        if (e != hipSuccess) return e;
        const long rows = (long)B * S * nh;
        k_attn_delta<D><<<(unsigned)((2 * rows + 255) / 256), 256, 0, st>>>((const bf16_t*)o, (const bf16_t*)dout, dvec, S, nh, rows);
        k_attn_bwd_both<D><<<grid + grid_kv, KVTHREADS, LDS_KV, st>>>((const bf16_t*)qkv, ld, bytes, (const bf16_t*)dout, do_bytes, lse, dvec,
                                                                      (bf16_t*)dqkv, S, nh, nkv, B, hs, scratch, rope, rope_seq);
    } else {
        constexpr int LDS = 4 * Tile<D>::BYTES;
        e = set_lds(k_attn_bwd_dq<D, 1>, LDS);
        if (e != hipSuccess) return e;
        k_attn_bwd_dq<D, 1><<<grid, ATHREADS, LDS, st>>>((const bf16_t*)qkv, ld, bytes, (const bf16_t*)o, (const bf16_t*)dout, do_bytes, lse, dvec,
                                                         (bf16_t*)dqkv, S, nh, nkv, B, rope, rope_seq);
        k_attn_bwd_dkv<D><<<grid_kv, KVTHREADS, LDS_KV, st>>>((const bf16_t*)qkv, ld, bytes, (const bf16_t*)dout, do_bytes, lse,
                                                              dvec, (bf16_t*)dqkv, S, nh, nkv, B, hs, scratch, rope, rope_seq);
    }
    if (hs > 1) {
        const long n = (long)B * S * (nkv * D / 8);
        k_attn_dkv_reduce<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(scratch, hs, (long)B * S, nkv * D, D, S, (bf16_t*)dqkv, ld, nh * D,
                                                                       rope, rope_seq);
    }
    return hipGetLastError();
}

hipError_t attn_bf16_fwd(const void* qkv, int ld, void* o, float* lse, int B, int S, int nh, int nkv, int d, hipStream_t st) {
    const long bytes = (long)B * S * ld * 2;
    if (bytes >= (1L << 32) - (1L << 25)) return hipErrorInvalidValue;
    if (d == 128) return fwd_d<128>(qkv, ld, (uint32_t)bytes, o, lse, B, S, nh, nkv, st);
    if (d == 64) return fwd_d<64>(qkv, ld, (uint32_t)bytes, o, lse, B, S, nh, nkv, st);
    return hipErrorInvalidValue;
}

hipError_t attn_bf16_bwd(const void* qkv, int ld, const void* o, const void* dout, const float* lse, float* dvec,
                         void* dqkv, float* scratch, int B, int S, int nh, int nkv, int d,
                         const float* rope, int rope_seq, hipStream_t st) {
    const long bytes = (long)B * S * ld * 2;
    const long do_bytes = (long)B * S * nh * d * 2;
    if (bytes >= (1L << 32) - (1L << 25)) return hipErrorInvalidValue;
    if (rope && rope_seq < S) return hipErrorInvalidValue;
    if (d == 128) return bwd_d<128>(qkv, ld, (uint32_t)bytes, o, dout, (uint32_t)do_bytes, lse, dvec, dqkv, scratch, B, S, nh, nkv, rope, rope_seq, st);
    if (d == 64) return bwd_d<64>(qkv, ld, (uint32_t)bytes, o, dout, (uint32_t)do_bytes, lse, dvec, dqkv, scratch, B, S, nh, nkv, rope, rope_seq, st);
    return hipErrorInvalidValue;
}

}  // namespace hh
