// bf16 x bf16 -> fp32 GEMMs on the gfx950 matrix cores for the projections of the
// decoder layer and their input / weight gradients.
//
//   NT  C[M,N] = A[M,K] B[N,K]^T      forward  y  = x W^T
//   NN  C[M,N] = A[M,K] B[K,N]        backward dX = dY W
//   TN  C[M,N] = A[K,M]^T B[K,N]      backward dW = dY^T X   (fp32 output, optional +=)
//
// Two kernels, both on v_mfma_f32_32x32x16_bf16:
//   * k_gemm_dma: 256x256 tile of C per workgroup of 8 waves (2 per SIMD, each a 128x64
//     sub-tile), k advancing 64 at a time through two LDS stages that are filled straight
//     from global memory (buffer_load ... lds), so a k-contiguous operand row is fetched as
//     one whole 128-byte line per stage.  The loop is laid out by hand: MFMAs of one k step
//     interleaved with the LDS fragment reads of the next, one barrier per stage placed
//     before its last k step, after which the other stage's first fragments and the DMA of
//     the stage after that are issued.
//   * k_gemm_bf16: 128x128 tile per workgroup of 4 waves, register-staged double buffer,
//     for problems too small to fill the chip with 256x256 tiles.
//
// Operand tiles in LDS keep the layout they have in memory, so global->LDS traffic is
// 16 bytes per lane with no transposition:
//   * k contiguous in memory  -> LDS [row][k], 16-byte chunks XOR-swizzled by the row
//     index; fragments come out with ds_read_b128.
//   * k strided in memory     -> LDS [k][rows], 64-byte slots XOR-swizzled by the k
//     index; fragments come out with the transposing ds_read_b64_tr_b16.
// Either way lane l of a fragment holds row (l % 32), k = 16*step + 8*(l/32) .. +7.
// Rows past the end of a tensor read as zero (buffer bounds), so ragged token counts
// need no special path.
//
// The MFMA takes the B-side fragment as its first operand, so each accumulator lane owns
// one row m of C and runs of 4 consecutive columns n: stores are 8-byte (bf16) or 16-byte
// (fp32) vectors along the contiguous dimension of C.
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
__device__ __forceinline__ void tile_of_index(int id, int tiles_m, int tiles_n, int& tm, int& tn) {
    const int nb = tiles_m * tiles_n;
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
    tile_of_index(blockIdx.x, (M + BM - 1) / BM, (N + BN - 1) / BN, tm, tn);
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
    static std::atomic<uint64_t> lds_ok{0};
    auto kern = k_gemm_bf16<KIND, BM, BN, OUT_F32>;
    const hipError_t e = allow_lds((const void*)kern, LDS, lds_ok);
    if (e != hipSuccess) return e;
    const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
    kern<<<tiles, GTHREADS, LDS, st>>>((const bf16_t*)g.A, g.lda, a_bytes, (const bf16_t*)g.B, g.ldb, b_bytes, g.C, g.ldc,
                                       (const bf16_t*)g.R, g.ldr, g.M, g.N, g.K, g.accumulate);
    return hipGetLastError();
}


// ---------------------------------------------------------------------------
// Large-tile kernel: 256x256 tile of C, k advances 64 at a time through TWO LDS
// stages that are filled straight from global memory (buffer_load ... lds: no
// VGPR staging, no ds_write).  A k-contiguous operand row is 128 bytes per stage,
// i.e. one full cache line per request.
constexpr int DK = 64;           // k per stage
constexpr int DSTAGES = 2;
constexpr int DTILE = 256;
constexpr int DSTAGE_BYTES = DTILE * DK * 2;   // one operand, one stage: 32 KB
// Of the 8 DMA instructions a wave issues per stage, the last DMA_LATE wait until k step 0 of the next stage
// (their buffer is free from the barrier on and the data is not needed before the next barrier): spreading the
// requests measured 1.2 % faster on a whole layer than issuing all 8 during k step 3; more, or later, was slower.
constexpr int DMA_LATE = 3;

__device__ __forceinline__ void dma16(uint32_t lds_addr, uint32_t voff, i32x4 rs) {
    // each lane moves 16 bytes from (rs.base + voff) to LDS byte (lds_addr + 16*lane); lanes past the
    // buffer's extent deposit zeros
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voff), "s"(rs) : "memory");
}

template <bool KC>
struct DmaTile {
    // Per wave and stage: 4 instructions of 1 KB (8 waves).  Instruction i of wave w covers
    //   KC : rows 8*(4w+i) .. +7     (128 B per row, lane -> row L/8, physical chunk L%8)
    //   KS : k rows 2*(4w+i), +1     (512 B per k row, lane -> k row L/32, physical chunk L%32)
    // The global address picks the logical chunk that the swizzle places at that physical slot.
    __device__ static __forceinline__ uint32_t voff(int i, int row0, int ld) {
        const int w = threadIdx.x >> 6, L = threadIdx.x & 63;
        if (KC) {
            const int r = 8 * (4 * w + i) + (L >> 3);
            const int logical = (L & 7) ^ ((r >> 1) & 7);
            return ((uint32_t)(row0 + r) * (uint32_t)ld + (uint32_t)(logical * 8)) * 2u;
        } else {
            const int k = 2 * (4 * w + i) + (L >> 5);
            const int lbyte = ((L & 31) * 16) ^ ((k & 3) << 6);
            return ((uint32_t)k * (uint32_t)ld + (uint32_t)row0) * 2u + (uint32_t)lbyte;
        }
    }
    __device__ static __forceinline__ uint32_t kstep_bytes(int ld) { return KC ? DK * 2u : (uint32_t)DK * (uint32_t)ld * 2u; }
    // fragment of 32 rows starting at rb, k step kk (0..3)
    __device__ static __forceinline__ bf16x8 frag(const char* lds, int rb, int kk) {
        const int l = threadIdx.x & 63;
        if (KC) {
            const int r = rb + (l & 31), c = 2 * kk + (l >> 5);
            return *reinterpret_cast<const bf16x8*>(lds + r * 128 + ((c ^ ((r >> 1) & 7)) << 4));
        } else {
            typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
            const int col = rb + 16 * ((l >> 4) & 1) + 4 * (l & 3);
            const int kr0 = 16 * kk + 8 * (l >> 5) + ((l & 15) >> 2);
            const int kr1 = kr0 + 4;
            const char* p0 = lds + kr0 * (DTILE * 2) + ((col * 2) ^ ((kr0 & 3) << 6));
            const char* p1 = lds + kr1 * (DTILE * 2) + ((col * 2) ^ ((kr1 & 3) << 6));
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p0);
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p1);
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    }
};

template <int KIND, bool OUT_F32>
__global__ __launch_bounds__(512) void k_gemm_dma(const bf16_t* __restrict__ A, int lda, uint32_t a_bytes,
                                                  const bf16_t* __restrict__ B, int ldb, uint32_t b_bytes,
                                                  void* __restrict__ Cv, int ldc, const bf16_t* R, int ldr,
                                                  int M, int N, int K, int accumulate,
                                                  int full, int n_items, int ksplit, float* __restrict__ partial) {
    // The workgroup walks work items blockIdx.x, + gridDim.x, ... < n_items.  Items below `full` are whole tiles
    // (all of k, written out through the epilogue).  Item full + q is the (q % ksplit)-th share of the k range of
    // tile full + q / ksplit; its fp32 sums go to partial[q][256][256] and k_splitk_reduce finishes those tiles.
    // The first DMA stages of the next item are issued before the current one is written out.
    constexpr bool A_KC = (KIND != GEMM_TN);
    constexpr bool B_KC = (KIND == GEMM_NT);
    using DA = DmaTile<A_KC>;
    using DB = DmaTile<B_KC>;
    constexpr int TM = 4, TN = 2;
    extern __shared__ __attribute__((aligned(1024))) char smem[];   // [stage][A 32 KB | B 32 KB]

    const int tiles_m = (M + DTILE - 1) / DTILE, tiles_n = (N + DTILE - 1) / DTILE;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5;
    const int wm = (wave >> 2) * 128, wn = (wave & 3) * 64;
    const int nk_all = (K + DK - 1) / DK;
    // work item -> tile index, first k tile, number of k tiles, slot in `partial` (-1: whole tile)
    int tix, kbeg, nk, slot;
    auto decode = [&](int item) {
        if (item < full) { tix = item; kbeg = 0; nk = nk_all; slot = -1; }
        else {
            const int q = item - full, chunk = q % ksplit;
            tix = full + q / ksplit;
            kbeg = (int)((long)chunk * nk_all / ksplit);
            nk = (int)((long)(chunk + 1) * nk_all / ksplit) - kbeg;
            slot = q;
        }
    };
    int item = (int)blockIdx.x;
    decode(item);

    const uint64_t pa = (uint64_t)A, pb = (uint64_t)B;
    const i32x4 rsA = {(int)(uint32_t)pa, (int)(uint32_t)(pa >> 32), (int)a_bytes, 0x00020000};
    const i32x4 rsB = {(int)(uint32_t)pb, (int)(uint32_t)(pb >> 32), (int)b_bytes, 0x00020000};
    uint32_t voA[4], voB[4];
    const uint32_t stepA = DA::kstep_bytes(lda), stepB = DB::kstep_bytes(ldb);
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;   // LDS byte address of the dynamic segment
    const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds0 + wave * 4096);

    constexpr uint32_t CES = OUT_F32 ? 4u : 2u;
    constexpr uint32_t OUT_OF_RANGE = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rsC = make_rsrc(Cv, (uint32_t)(((size_t)(M - 1) * ldc + N) * CES));
    const __amdgpu_buffer_rsrc_t rsR = make_rsrc(R ? (const void*)R : (const void*)Cv, R ? (uint32_t)(((size_t)(M - 1) * ldr + N) * 2u) : 0u);

#define SB() __builtin_amdgcn_sched_barrier(0)
    // one DMA instruction of the k tile being issued (i < 4: A part i, else B part i-4) into stage st
    auto dma_part = [&](int st, int i) {
        const uint32_t base = wave_lds + st * (2 * DSTAGE_BYTES);
        if (i < 4) { dma16(base + i * 1024, voA[i], rsA); voA[i] += stepA; }
        else { dma16(base + DSTAGE_BYTES + (i - 4) * 1024, voB[i - 4], rsB); voB[i - 4] += stepB; }
    };
    // point the DMA offsets at tile (m0, n0) and put its first two k tiles on their way
    auto start_tile = [&](int m0, int n0) {
#pragma unroll
        for (int i = 0; i < 4; i++) { voA[i] = DA::voff(i, m0, lda) + kbeg * stepA; voB[i] = DB::voff(i, n0, ldb) + kbeg * stepB; }
#pragma unroll
        for (int s = 0; s < 2; s++)
            if (s < nk) {
#pragma unroll
                for (int i = 0; i < 8; i++) dma_part(s, i);
            }
    };

    int tm, tn;
    tile_of_index(tix, tiles_m, tiles_n, tm, tn);
    int m0 = tm * DTILE, n0 = tn * DTILE;
    start_tile(m0, n0);
    bool fresh = true;   // no stores of an earlier tile are in flight behind the DMAs

    for (;;) {
        f32x16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
            for (int j = 0; j < TN; j++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

        // k tile 0 landed.  After an epilogue its stores sit behind the DMAs in the memory queue, so the
        // count-based wait only applies to a fresh start.
        if (fresh && nk > 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        bf16x8 a0[TM], b0[TN], a1[TM], b1[TN];
#pragma unroll
        for (int i = 0; i < TM; i++) a0[i] = DA::frag(smem, wm + 32 * i, 0);
#pragma unroll
        for (int j = 0; j < TN; j++) b0[j] = DB::frag(smem + DSTAGE_BYTES, wn + 32 * j, 0);

        for (int kt = 0; kt < nk; kt++) {
            const char* cA = smem + (kt & 1) * (2 * DSTAGE_BYTES);
            const char* cB = cA + DSTAGE_BYTES;
            const char* nA = smem + ((kt + 1) & 1) * (2 * DSTAGE_BYTES);
            const char* nB = nA + DSTAGE_BYTES;
            const bool more = kt + 2 < nk;
            const bool late = kt >= 1 && kt + 1 < nk;   // k tile kt+1's last DMA instructions are still to be issued
            SB();
            // k steps 0..2 of tile kt: MFMAs on one fragment set while the next one is fetched
#pragma unroll
            for (int kk = 0; kk < 3; kk++) {
                bf16x8 (&ca)[TM] = (kk & 1) ? a1 : a0;
                bf16x8 (&cb)[TN] = (kk & 1) ? b1 : b0;
                bf16x8 (&na)[TM] = (kk & 1) ? a0 : a1;
                bf16x8 (&nb)[TN] = (kk & 1) ? b0 : b1;
#pragma unroll
                for (int i = 0; i < TM; i++) {
#pragma unroll
                    for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cb[j], ca[i], acc[i][j], 0, 0, 0);
                    if (i == 0) { na[0] = DA::frag(cA, wm, kk + 1); nb[0] = DB::frag(cB, wn, kk + 1); nb[1] = DB::frag(cB, wn + 32, kk + 1); }
                    if (i == 1) { na[1] = DA::frag(cA, wm + 32, kk + 1); na[2] = DA::frag(cA, wm + 64, kk + 1); }
                    if (i == 2) { na[3] = DA::frag(cA, wm + 96, kk + 1); }
                    if (kk == 0 && i < DMA_LATE && late) dma_part((kt + 1) & 1, 8 - DMA_LATE + i);
                    SB();
                }
            }
            // Every wave now holds its last fragments of tile kt, so the stage of tile kt is free once all
            // waves are here; tile kt+1 (issued one tile ago) must have landed for everyone.
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            SB();
            // k step 3: MFMAs on (a1, b1); meanwhile fetch the first fragments of tile kt+1 and issue most of tile kt+2
#pragma unroll
            for (int i = 0; i < TM; i++) {
#pragma unroll
                for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1[j], a1[i], acc[i][j], 0, 0, 0);
                if (i == 0) { a0[0] = DA::frag(nA, wm, 0); b0[0] = DB::frag(nB, wn, 0); b0[1] = DB::frag(nB, wn + 32, 0); }
                if (i == 1) { a0[1] = DA::frag(nA, wm + 32, 0); a0[2] = DA::frag(nA, wm + 64, 0); }
                if (i == 2) { a0[3] = DA::frag(nA, wm + 96, 0); }
                if (more) {
#pragma unroll
                    for (int q = 0; q < 8 - DMA_LATE; q++)
                        if (q * 4 / (8 - DMA_LATE) == i) dma_part(kt & 1, q);
                }
                SB();
            }
        }

        // next piece of work of this workgroup: start its loads before writing this one out
        const int cm0 = m0, cn0 = n0, cacc = accumulate, cslot = slot;
        item += (int)gridDim.x;
        const bool has_next = item < n_items;
        if (has_next) {
            decode(item);
            tile_of_index(tix, tiles_m, tiles_n, tm, tn);
            m0 = tm * DTILE; n0 = tn * DTILE;
            __syncthreads();   // every wave has finished reading the LDS stages
            start_tile(m0, n0);
            fresh = false;
        }

        if (cslot >= 0) {   // a share of the k range: raw fp32 sums, finished by the reduction kernel
            float* pt = partial + (size_t)cslot * (DTILE * DTILE);
#pragma unroll
            for (int i = 0; i < TM; i++)
#pragma unroll
                for (int j = 0; j < TN; j++)
#pragma unroll
                    for (int g = 0; g < 4; g++)
                        *reinterpret_cast<float4*>(pt + (wm + 32 * i + (lane & 31)) * DTILE + wn + 32 * j + 8 * g + 4 * hf) =
                            make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
            if (!has_next) return;
            continue;
        }

        // Epilogue.  In the accumulators a lane owns one row and 4-column pieces of it, which would make every
        // store instruction touch 32 rows with 16 or 32 bytes each.  Each 32x32 block therefore goes through a
        // wave-private 4 KB LDS patch (fp32, 16-byte chunks XOR-swizzled by the row) and comes back with 8
        // lanes per row: loads of what is added (old fp32 sums or the bf16 residual) and stores then cover
        // whole 128-byte (fp32) or 64-byte (bf16) row segments.  C and R are reached through bounds-checked
        // buffers: rows past M fall behind the buffer's end, columns past N get an out-of-range offset.
        {
            char* const patch = smem + DSTAGES * 2 * DSTAGE_BYTES + wave * 4096;
            const int r_w = lane & 31;                       // row written, chunks 2g + hf
            const int r_r = lane >> 3, c_r = lane & 7;       // row (+ 8t) and chunk read back
#pragma unroll
            for (int i = 0; i < TM; i++) {
                const uint32_t row_base = (uint32_t)(cm0 + wm + 32 * i + r_r);
                float4 add[TN][4];
                uint32_t off_c[TN][4];
#pragma unroll
                for (int j = 0; j < TN; j++) {
                    const int col = cn0 + wn + 32 * j + 4 * c_r;
#pragma unroll
                    for (int t = 0; t < 4; t++) {
                        const uint32_t row = row_base + 8 * t;
                        off_c[j][t] = col < N ? (row * (uint32_t)ldc + (uint32_t)col) * CES : OUT_OF_RANGE;
                        add[j][t] = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (OUT_F32) {
                            if (cacc) {
                                const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsC, off_c[j][t], 0, 0);
                                add[j][t] = make_float4(__int_as_float(v[0]), __int_as_float(v[1]), __int_as_float(v[2]), __int_as_float(v[3]));
                            }
                        } else if (R) {
                            const uint32_t off_r = col < N ? (row * (uint32_t)ldr + (uint32_t)col) * 2u : OUT_OF_RANGE;
                            const i32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsR, off_r, 0, 0);
                            add[j][t] = make_float4(lo_bf((uint32_t)v[0]), hi_bf((uint32_t)v[0]), lo_bf((uint32_t)v[1]), hi_bf((uint32_t)v[1]));
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < TN; j++) {
#pragma unroll
                    for (int g = 0; g < 4; g++)
                        *reinterpret_cast<float4*>(patch + r_w * 128 + (((2 * g + hf) ^ ((r_w >> 1) & 7)) << 4)) =
                            make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
#pragma unroll
                    for (int t = 0; t < 4; t++) {
                        const int rr = 8 * t + r_r;
                        float4 v = *reinterpret_cast<const float4*>(patch + rr * 128 + ((c_r ^ ((rr >> 1) & 7)) << 4));
                        v.x += add[j][t].x; v.y += add[j][t].y; v.z += add[j][t].z; v.w += add[j][t].w;
                        if (OUT_F32) {
                            const i32x4 o = {__float_as_int(v.x), __float_as_int(v.y), __float_as_int(v.z), __float_as_int(v.w)};
                            __builtin_amdgcn_raw_buffer_store_b128(o, rsC, off_c[j][t], 0, 0);
                        } else {
                            const i32x2 o = {(int)pack_bf2(v.x, v.y), (int)pack_bf2(v.z, v.w)};
                            __builtin_amdgcn_raw_buffer_store_b64(o, rsC, off_c[j][t], 0, 0);
                        }
                    }
                }
            }
        }
        if (!has_next) return;
    }
#undef SB
}

// Sums the ksplit fp32 partial tiles of each split tile in a fixed order and applies the epilogue.
// 64 workgroups per tile; a thread owns 4 consecutive columns of one row.
template <bool OUT_F32>
__global__ __launch_bounds__(256) void k_splitk_reduce(const float* __restrict__ partial, int ksplit, int block0,
                                                       void* __restrict__ Cv, int ldc, const bf16_t* R, int ldr,
                                                       int M, int N, int accumulate) {
    const int r = blockIdx.x >> 6, sub = blockIdx.x & 63;
    int tm, tn;
    tile_of_index(block0 + r, (M + DTILE - 1) / DTILE, (N + DTILE - 1) / DTILE, tm, tn);
    const int q = sub * 256 + threadIdx.x;
    const int row = q >> 6, col = (q & 63) * 4;
    const float* p = partial + (size_t)r * ksplit * (DTILE * DTILE) + row * DTILE + col;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < ksplit; c++) {
        const float4 t = *reinterpret_cast<const float4*>(p + (size_t)c * (DTILE * DTILE));
        v[0] += t.x; v[1] += t.y; v[2] += t.z; v[3] += t.w;
    }
    const int m = tm * DTILE + row, n = tn * DTILE + col;
    if (m >= M || n >= N) return;
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

// Compute units of the current device (one persistent workgroup each), asked once per device.
static int device_cus(hipError_t& err) {
    static std::atomic<int> cached[64];
    int dev = 0;
    err = hipGetDevice(&dev);
    if (err != hipSuccess) return 0;
    const int slot = dev & 63;
    int n = cached[slot].load(std::memory_order_relaxed);
    if (n > 0) return n;
    err = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (err != hipSuccess) return 0;
    if (n < 8) n = 8;
    cached[slot].store(n, std::memory_order_relaxed);
    return n;
}

// Full rounds of one tile per compute unit run as one persistent workgroup per unit.  A last, partial round of R
// tiles would leave most units idle, so it is cut along k into floor(units / R) shares per tile, which the same
// workgroups take up after their whole tiles (fp32 partials in `ws`, summed in a fixed order by a small second kernel).
template <int KIND, bool OUT_F32>
static hipError_t launch_dma(const GemmDesc& g, uint32_t a_bytes, uint32_t b_bytes, hipStream_t st) {
    constexpr int LDS = DSTAGES * 2 * DSTAGE_BYTES + 8 * 4096;   // two stages + the epilogue patches of the 8 waves
    static std::atomic<uint64_t> lds_ok{0};
    auto kern = k_gemm_dma<KIND, OUT_F32>;
    const hipError_t e = allow_lds((const void*)kern, LDS, lds_ok);
    if (e != hipSuccess) return e;
    hipError_t ce = hipSuccess;
    const int NUM_CU = device_cus(ce);
    if (ce != hipSuccess) return ce;
    const int tiles = ((g.M + DTILE - 1) / DTILE) * ((g.N + DTILE - 1) / DTILE);
    const int nk = (g.K + DK - 1) / DK;
    int full = tiles, tail = 0, ksplit = 1;
    const int rem = tiles % NUM_CU;
    if (rem > 0 && rem <= NUM_CU / 2 && g.ws) {
        int s = NUM_CU / rem;
        if (s > 8) s = 8;
        while (s > 1 && (nk / s < 4 || (size_t)rem * s * DTILE * DTILE * sizeof(float) > g.ws_bytes)) s--;
        if (s > 1) { full = tiles - rem; tail = rem; ksplit = s; }
    }
    // one launch: a persistent workgroup per CU walks the whole tiles and then the k shares of the tail tiles
    const int n_items = full + tail * ksplit;
    kern<<<n_items < NUM_CU ? n_items : NUM_CU, 512, LDS, st>>>((const bf16_t*)g.A, g.lda, a_bytes, (const bf16_t*)g.B, g.ldb, b_bytes,
                                                                 g.C, g.ldc, (const bf16_t*)g.R, g.ldr, g.M, g.N, g.K, g.accumulate,
                                                                 full, n_items, ksplit, (float*)g.ws);
    if (tail > 0)
        k_splitk_reduce<OUT_F32><<<tail * 64, 256, 0, st>>>((const float*)g.ws, ksplit, full, g.C, g.ldc, (const bf16_t*)g.R,
                                                            g.ldr, g.M, g.N, g.accumulate);
    return hipGetLastError();
}

template <int KIND, bool OUT_F32>
static hipError_t pick_tile(const GemmDesc& g, uint32_t a_bytes, uint32_t b_bytes, hipStream_t st) {
    // 256x256 tiles (k-split when they are few) unless the problem is small; 128x128 tiles otherwise
    const long big = (long)((g.M + 255) / 256) * ((g.N + 255) / 256);
    if (big >= 64) return launch_dma<KIND, OUT_F32>(g, a_bytes, b_bytes, st);
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
    // C (and the residual) are addressed with 32-bit byte offsets below 2 GB
    if (((long)(g.M - 1) * g.ldc + g.N) * (g.out_f32 ? 4 : 2) >= (1L << 31)) return hipErrorInvalidValue;
    if (g.R && ((long)(g.M - 1) * g.ldr + g.N) * 2 >= (1L << 31)) return hipErrorInvalidValue;
    // a k-contiguous operand is fetched 64 k values at a time with no per-row bound
    if (g.kind != GEMM_TN && g.K % 64 != 0) return hipErrorInvalidValue;
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
