// Host-side launchers of the gfx950 kernels (internal to the library).
// All pointers are device pointers; every launcher only enqueues on `st`.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace hh {

enum { DT_F32 = 0, DT_BF16 = 1 };
inline size_t dt_size(int dt) { return dt == DT_BF16 ? 2 : 4; }

// C[M,N] (=|+=) op(A) op(B) (+ R), leading dimensions in elements.
//   GEMM_NT: A[M,K] row-major, B[N,K] row-major   (y = x W^T)
//   GEMM_NN: A[M,K] row-major, B[K,N] row-major   (dX = dY W)
//   GEMM_TN: A[K,M] row-major, B[K,N] row-major   (dW = dY^T X)
enum { GEMM_NT = 0, GEMM_NN = 1, GEMM_TN = 2 };
struct GemmDesc {
    int kind;
    int M, N, K;
    const void* A; int lda;
    const void* B; int ldb;
    void* C; int ldc;
    const void* R; int ldr;  // optional residual in the storage dtype, added before rounding (NULL: none)
    int out_f32;             // 1: C is fp32 regardless of the storage dtype (parameter gradients)
    int accumulate;          // 1: C += result
    void* ws;                // optional scratch for k-split partial sums (bf16 path), may be NULL
    size_t ws_bytes;
};
constexpr size_t GEMM_WS_BYTES = (size_t)64 << 20;   // enough for 256 partial tiles of 256x256 fp32

// The library's own scratch array (one per GPU, held until the process ends) and its size.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)128 << 20;
hipError_t static_scratch_init(int device);   // `device` must be current; looks the array's address up once
void* static_scratch(int device);             // that address (null before a successful init)
hipError_t gemm(int dtype, const GemmDesc& g, hipStream_t st);

// xn = x * r * g, r = 1/sqrt(mean(x^2)+eps) per row.
hipError_t rmsnorm_fwd(int dtype, const void* x, const void* g, void* xn, float* r,
                       int T, int H, float eps, hipStream_t st);
// dx = dres + r*(w - u*mean(w*u)), u = x*r, w = dxn*g; per-workgroup column sums of
// dxn*u go to partial[rmsnorm_bwd_blocks(T), H].
int rmsnorm_bwd_blocks(int T);
hipError_t rmsnorm_bwd(int dtype, const void* dxn, const void* x, const float* r, const void* g,
                       const void* dres, void* dx, float* partial, int T, int H, hipStream_t st);
hipError_t colsum_reduce(const float* partial, int nblk, int H, float* out, int accumulate, hipStream_t st);

// In-place rotary embedding of the first nrot heads (query heads, then key heads) of every row of a
// [T, ld] buffer.  table = cos[table_seq][d/2] followed by sin[table_seq][d/2], table_seq >= S.
// backward: rotate by -angle.
hipError_t rope(int dtype, void* qkv, int ld, int T, int S, int nrot, int d, const float* table, int table_seq,
                int backward, hipStream_t st);

// gu[T,2F] = (gate | up);  m = silu(gate)*up
hipError_t swiglu_fwd(int dtype, const void* gu, void* m, int T, int F, hipStream_t st);
// dgu[T,2F] = (dgate | dup), and m recomputed
hipError_t swiglu_bwd(int dtype, const void* dm, const void* gu, void* dgu, void* m, int T, int F, hipStream_t st);

// Causal attention over a [T, ld] buffer holding q | k | v column blocks of width nh*d, nkv*d, nkv*d;
// query head h uses key/value head h / (nh / nkv).  o [T, nh*d]; lse [B, nh, S] natural-log sum-exp of
// the scaled scores.
hipError_t attn_fwd(int dtype, const void* qkv, int ld, void* o, float* lse,
                    int B, int S, int nh, int nkv, int d, hipStream_t st);
// dqkv [T, ld] receives dq | dk | dv in the same layout.  dvec: scratch [B, nh, S] floats.  scratch: device
// memory of attn_bwd_scratch_bytes() bytes (partial dK, dV sums when the query heads that share a key/value head
// are spread over several workgroups; may be null when that size is 0).  rope_table (as for rope(), rope_seq >= S;
// null: none): q and k were rotated before the forward call, and dq, dk are written as gradients of the
// unrotated q, k (the backward rotation applied before the one rounding to the storage type).
size_t attn_bwd_scratch_bytes(int dtype, int B, int S, int nh, int nkv, int d);
hipError_t attn_bwd(int dtype, const void* qkv, int ld, const void* o, const void* dout, const float* lse,
                    float* dvec, void* dqkv, void* scratch, int B, int S, int nh, int nkv, int d,
                    const float* rope_table, int rope_seq, hipStream_t st);

}  // namespace hh
