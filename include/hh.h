/* hh.h -- C ABI of the per-GPU pipeline-stage step of a Llama-style model.
 *
 * Scope.  In hybrid-parallel training each accelerator owns a pipeline stage of
 * 1..k consecutive transformer layers and processes the batch as micro-batches
 * (paper Section 2.3); its run time is the forward and backward pass of those
 * layers.  This library is that per-device work for Llama2 decoder layers (the
 * model family of Section 4.2 / Table 1) on one gfx950 GPU: hand-written HIP
 * kernels only.  The per-layer timings it exports are the "computation
 * performance of the operator or layer" that the performance predictor of
 * Section 3.2 samples from each accelerator type.
 *
 * Layer (pre-norm Llama decoder layer, no bias, no dropout), T = micro_batch*seq
 * tokens, H hidden, A = n_heads*head_dim, Akv = n_kv_heads*head_dim, F = ffn:
 *     xn = rmsnorm(x; g_attn)          q,k,v = xn Wq^T, xn Wk^T, xn Wv^T
 *     q,k <- rope(q), rope(k)          (pairs (i, i+head_dim/2), angle pos*base^(-2i/d))
 *     a  = causal_softmax(q k^T / sqrt(d)) v      per (sample, query head); query head h reads key/value
 *                                                 head h / (n_heads / n_kv_heads)  (grouped-query attention)
 *     h  = x + a Wo^T                  hn = rmsnorm(h; g_mlp)
 *     y  = h + (silu(hn Wg^T) * (hn Wu^T)) Wd^T
 * rmsnorm(t; g) = t * g / sqrt(mean(t^2) + rms_eps).  When the shapes are one
 * tensor-parallel share (A != H), a Wo^T and m Wd^T are that share's partial
 * sums and are added to the residual as they are: the all-reduce between
 * shares is not part of this library.
 *
 * General rules
 *  - Every function returns HH_OK (0) or a negative hh_status; none aborts,
 *    throws or prints.  hh_last_error() gives a message for the calling thread.
 *  - All tensor pointers are DEVICE pointers unless a parameter says "host".
 *    The caller owns every buffer; the hot calls (hh_layer_fwd, hh_layer_bwd,
 *    hh_stage_step) allocate nothing except, once per context, the rotary
 *    cos/sin table for a new (seq, head_dim, rope_base); hh_ctx_reserve does
 *    that ahead of time.
 *  - The hot calls enqueue work on `stream` (a hipStream_t passed as void*,
 *    NULL = the null stream) and return without synchronising.
 *  - Layouts: activations [micro_batch, seq, feat] row-major contiguous;
 *    weights [out, in] row-major.  dtype HH_BF16: activations and weights are
 *    bfloat16, accumulation fp32, parameter gradients fp32.  dtype HH_F32:
 *    everything fp32.
 *  - Every pointer must be 16-byte aligned (HH_ERR_MISALIGNED otherwise).
 *  - Shapes: head_dim 64 or 128; n_kv_heads divides n_heads; hidden, n_heads*head_dim
 *    and ffn multiples of 64 for HH_BF16 and multiples of 8 for HH_F32; any
 *    seq >= 1, micro_batch >= 1; every activation and every single fp32 gradient
 *    below 2^31 bytes, every (packed) weight below 2^32 - 2^25 bytes
 *    (HH_ERR_UNSUPPORTED_SHAPE otherwise).
 *  - Argument validation happens before any GPU work is enqueued.
 *  - A context is used by one host thread at a time (the hot calls keep per-call state in it); use one context
 *    per thread.  A rotary table that a later call replaces by a longer one stays alive until hh_ctx_destroy,
 *    so work enqueued or captured earlier keeps reading valid memory.
 */
#ifndef HH_H
#define HH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HH_OK = 0,
    HH_ERR_INVALID_ARG = -1,       /* null pointer, non-positive count, bad enum */
    HH_ERR_UNSUPPORTED_SHAPE = -2, /* see "Shapes" above */
    HH_ERR_BUFFER_TOO_SMALL = -3,  /* hh_layer_fwd_noalloc: the shape needs more scratch than the library's array holds */
    HH_ERR_MISALIGNED = -4,
    HH_ERR_DEVICE = -5             /* a HIP runtime call failed; text in hh_last_error() */
} hh_status;

typedef enum { HH_F32 = 0, HH_BF16 = 1 } hh_dtype;

/* Shape of one decoder layer and of the micro-batch it processes. */
typedef struct {
    int32_t hidden;       /* H */
    int32_t n_heads;      /* heads held by this GPU */
    int32_t n_kv_heads;   /* divides n_heads; query head h uses key/value head h / (n_heads / n_kv_heads) */
    int32_t head_dim;     /* d: 64 or 128 */
    int32_t ffn;          /* F: SwiGLU width held by this GPU */
    int32_t seq;          /* S */
    int32_t micro_batch;  /* B: samples per micro-batch */
    float rms_eps;        /* inside the square root, added to the mean of squares */
    float rope_base;
    int32_t dtype;        /* hh_dtype */
} hh_layer_cfg;

/* Parameters of one layer, in the storage dtype.  wq, wk, wv may be three row
 * blocks of one [A + 2*Akv, H] allocation, w_gate and w_up of one [2F, H]
 * allocation: the library then runs one GEMM instead of three / two. */
typedef struct {
    const void *g_attn;  /* [H]    */
    const void *wq;      /* [A, H] */
    const void *wk;      /* [Akv, H] */
    const void *wv;      /* [Akv, H] */
    const void *wo;      /* [H, A] */
    const void *g_mlp;   /* [H]    */
    const void *w_gate;  /* [F, H] */
    const void *w_up;    /* [F, H] */
    const void *w_down;  /* [H, F] */
} hh_layer_weights;

/* Parameter gradients, always fp32, same shapes as the weights. */
typedef struct {
    float *g_attn, *wq, *wk, *wv, *wo, *g_mlp, *w_gate, *w_up, *w_down;
} hh_layer_grads;

/* One node of the predictor's weighted graph (Section 3.2): measured time of one
 * layer on this device plus the memory figures the workload simulator needs. */
typedef struct {
    int32_t layer;
    float fwd_ms, bwd_ms;          /* median over the timed iterations */
    double fwd_flop, bwd_flop;     /* model flops: GEMM 2mnk, causal attention 4*d per (query, key<=query) pair */
    float fwd_tflops, bwd_tflops;
    uint64_t weight_bytes;         /* parameters in the storage dtype */
    uint64_t grad_bytes;           /* fp32 parameter gradients */
    uint64_t saved_act_bytes;      /* activations kept from forward to backward, per micro-batch */
    uint64_t p2p_bytes;            /* stage-boundary message, Eq. (3): micro_batch*seq*hidden*2 */
    uint64_t workspace_bytes;      /* scratch one forward or backward pass of a layer needs (shared by all layers of a
                                      stage): with saved_act_bytes x live micro-batches x layers it gives the stage's
                                      activation high-water mark */
} hh_profile_rec;

typedef struct hh_ctx hh_ctx;      /* opaque: device id, rotary table */

/* Thread-local description of the last error on this thread ("" if none). */
const char *hh_last_error(void);

/* Create / destroy a context on HIP device `device`.  HH_ERR_DEVICE when there
 * is no such GPU.  Destroy frees the rotary tables; it does not synchronise: the
 * caller makes sure the work it enqueued with the context has finished. */
int hh_ctx_create(hh_ctx **out, int device);
int hh_ctx_destroy(hh_ctx *ctx);
/* Build the rotary table for cfg now (allocates and copies; a blocking host-to-device copy). */
int hh_ctx_reserve(hh_ctx *ctx, const hh_layer_cfg *cfg);

/* Model flops of one layer on one micro-batch (host arithmetic only). */
int hh_layer_flops(const hh_layer_cfg *cfg, double *fwd_flop, double *bwd_flop);

/* Bytes of the `saved` block of one layer x micro-batch and of the scratch
 * `workspace` that one fwd or bwd call needs (contents of workspace need not
 * survive between calls).  Host arithmetic only; validates cfg. */
int hh_layer_sizes(const hh_layer_cfg *cfg, size_t *saved_bytes, size_t *workspace_bytes);

/* Where each saved tensor of hh_layer_fwd sits inside the `saved` block (byte offsets from its start; the
 * tensors are the intermediate values of the layer equations at the top of this file).  xn, h, hn: [T, H];
 * qkv: [T, A + 2*Akv] rows of rotated q | rotated k | v; a: [T, A]; gate_up: [T, 2F] rows of gate | up (storage
 * dtype); lse: [B, n_heads, S] fp32, natural-log sum-exp of the scaled causal scores; r1, r2: [T] fp32, the
 * inverse RMS of x and of h.  total equals saved_bytes of hh_layer_sizes.  Host arithmetic only. */
typedef struct {
    size_t xn, qkv, a, h, hn, gate_up, lse, r1, r2, total;
} hh_saved_layout;
int hh_saved_layout_of(const hh_layer_cfg *cfg, hh_saved_layout *out);

/* Forward of one layer.  x [B,S,H] in, y [B,S,H] out (y must not alias x).
 * `saved` (>= saved_bytes) receives what backward needs besides x itself:
 * xn, rotated q and k, v, a, h, hn, gate, up, the softmax log-sum-exp and both
 * inverse RMS vectors.  saved == NULL runs forward only; workspace must then
 * hold saved_bytes + workspace_bytes. */
int hh_layer_fwd(hh_ctx *ctx, const hh_layer_cfg *cfg, const hh_layer_weights *w,
                 const void *x, void *y, void *saved, void *workspace, void *stream);

/* Forward of one layer for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as hh_layer_fwd(saved = NULL),
 * bit for bit; the scratch it needs (hh_layer_sizes: saved_bytes + workspace_bytes) is taken from an array of
 * HH_STATIC_SCRATCH_BYTES that the library holds on every GPU it is loaded on until the process ends.  The call makes
 * no allocation and no synchronisation: the rotary table must exist already (hh_ctx_reserve with a cfg of at least
 * this seq, same head_dim and rope_base; HH_ERR_INVALID_ARG otherwise), and a shape that needs more scratch than the
 * array holds is refused with HH_ERR_BUFFER_TOO_SMALL before anything is enqueued.  Every call on one GPU uses that
 * GPU's one array (nothing in it has to be cleared between calls; its contents are whatever the last call left):
 * two calls whose work overlaps in time on the same GPU, from any context or stream, race. */
#define HH_STATIC_SCRATCH_BYTES ((size_t)128 << 20)
int hh_layer_fwd_noalloc(hh_ctx *ctx, const hh_layer_cfg *cfg, const hh_layer_weights *w,
                         const void *x, void *y, void *stream);

/* Backward of one layer.  x and saved as given to / written by hh_layer_fwd;
 * dy [B,S,H] in; dx [B,S,H] out (dx may alias dy).  accumulate == 0 writes the
 * nine gradients, != 0 adds to them (fp32). */
int hh_layer_bwd(hh_ctx *ctx, const hh_layer_cfg *cfg, const hh_layer_weights *w,
                 const void *x, const void *saved, const void *dy, void *dx,
                 const hh_layer_grads *grads, int accumulate, void *workspace, void *stream);

/* Sizes for a stage of n_layers layers over n_micro micro-batches: the pool
 * keeps every layer's saved block and the activations between layers for all
 * micro-batches (forward of all micro-batches precedes backward). */
int hh_stage_sizes(const hh_layer_cfg *cfg, int n_layers, int n_micro,
                   size_t *saved_pool_bytes, size_t *workspace_bytes);

/* One pipeline-stage step (Section 2.3): for m in 0..n_micro-1 run x[m] through
 * layers 0..n_layers-1 into y[m]; then for m in 0..n_micro-1 run dy[m] back
 * through layers n_layers-1..0 into dx[m], summing parameter gradients over
 * micro-batches in fp32 (plain sum).  x, y, dy, dx are HOST arrays of n_micro
 * device pointers; w and g are HOST arrays of n_layers structs.
 * zero_grads_first != 0: the first micro-batch overwrites the gradients,
 * otherwise the step adds to what the buffers hold.  No allocation, no
 * synchronisation, no host-device copies. */
int hh_stage_step(hh_ctx *ctx, const hh_layer_cfg *cfg, int n_layers, const hh_layer_weights *w,
                  int n_micro, const void *const *x, void *const *y,
                  const void *const *dy, void *const *dx,
                  const hh_layer_grads *g, int zero_grads_first,
                  void *saved_pool, void *workspace, void *stream);

/* The same step in one-forward-one-backward order (PipeDream-1F1B, Section 2.3,
 * the scheme whose data constraints the pipeline of Section 3.3 keeps): forward
 * of micro-batches 0..n_live-1, then for m = 0..n_micro-1 backward of m followed
 * by forward of m + n_live.  At most n_live micro-batches' activations are alive,
 * so saved_pool is sized by hh_stage_sizes(cfg, n_layers, n_live): that figure
 * is the stage's activation high-water mark.  In a pipeline of P stages the
 * stage of rank r uses n_live = min(n_micro, P - r).  1 <= n_live <= n_micro;
 * n_live == n_micro is hh_stage_step.  Backward visits the micro-batches in
 * ascending order in both, so the results are bit-identical to hh_stage_step.
 * y[m + n_live] is written while dy[m + 1 ...] are still to be read: y and dy
 * arrays must not share buffers across micro-batches. */
int hh_stage_step_1f1b(hh_ctx *ctx, const hh_layer_cfg *cfg, int n_layers, const hh_layer_weights *w,
                       int n_micro, int n_live, const void *const *x, void *const *y,
                       const void *const *dy, void *const *dx, const hh_layer_grads *g,
                       int zero_grads_first, void *saved_pool, void *workspace, void *stream);

/* Time every layer of a stage (Sections 1 and 3.2: automatic profiling that
 * feeds the predictor).  Runs the stage on x / dy (device, [B,S,H]) with
 * `warmup` untimed and `iters` timed repetitions, bracketing each layer's
 * forward and backward with HIP events, and fills out[0..n_layers-1] (HOST).
 * Gradients are accumulated into g (values are meaningless afterwards).
 * saved_pool / workspace sized by hh_stage_sizes(cfg, n_layers, 1).
 * Synchronises the stream. */
int hh_layer_profile(hh_ctx *ctx, const hh_layer_cfg *cfg, int n_layers, const hh_layer_weights *w,
                     const hh_layer_grads *g, const void *x, const void *dy,
                     int warmup, int iters, void *saved_pool, void *workspace,
                     hh_profile_rec *out, void *stream);

/* Per-kernel-family timing of whatever the hot calls enqueue (the measurement
 * side of the automatic profiling of Section 3.2).  Between hh_trace_begin and
 * hh_trace_end every launch of a family whose bit (1u << kind) is set in
 * kind_mask is bracketed by HIP events on its stream, up to max_launches
 * launches (later ones are not recorded).  Events between kernels cost a few
 * microseconds each, so a caller that times a whole step selects only the
 * families it needs.  hh_trace_begin creates
 * the events (not a hot call); hh_trace_end waits for them and fills
 * out[0..n_kinds-1] (HOST) with launch count, summed milliseconds and summed
 * work: model flops for GEMM and attention families, algorithmic bytes for the
 * elementwise family. */
typedef enum {
    HH_TRACE_GEMM_NT = 0,      /* forward projections       y  = x W^T   */
    HH_TRACE_GEMM_NN = 1,      /* input gradients           dX = dY W    */
    HH_TRACE_GEMM_TN = 2,      /* weight gradients          dW = dY^T X  */
    HH_TRACE_ATTN_FWD = 3,
    HH_TRACE_ATTN_BWD = 4,
    HH_TRACE_ELEMENTWISE = 5,  /* RMSNorm, RoPE, SwiGLU, gain-gradient reduction */
    HH_TRACE_KINDS = 6
} hh_trace_kind;
typedef struct {
    int32_t kind;
    int32_t launches;
    double ms;
    double work;
} hh_trace_sum;
int hh_trace_begin(hh_ctx *ctx, int max_launches, uint32_t kind_mask);
int hh_trace_end(hh_ctx *ctx, hh_trace_sum *out, int n_kinds);

#ifdef __cplusplus
}
#endif
#endif /* HH_H */
