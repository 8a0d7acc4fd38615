// C ABI of the decoder-stage library: argument validation, buffer carving and
// the order in which the gfx950 kernels are enqueued.  No numeric work happens
// on the host except the rotary cos/sin table (built once per context).
#include "../../include/hh.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "kernels.h"

namespace hh {
hipError_t gemm_bf16(const GemmDesc& g, hipStream_t st);
hipError_t gemm_f32(const GemmDesc& g, hipStream_t st);
hipError_t attn_bf16_fwd(const void* qkv, int ld, void* o, float* lse, int B, int S, int nh, int nkv, int d, hipStream_t st);
hipError_t attn_bf16_bwd(const void* qkv, int ld, const void* o, const void* dout, const float* lse, float* dvec,
                         void* dqkv, float* scratch, int B, int S, int nh, int nkv, int d,
                         const float* rope, int rope_seq, hipStream_t st);
size_t attn_bf16_bwd_scratch_bytes(int B, int S, int nh, int nkv, int d);
hipError_t attn_f32_fwd(const void* qkv, int ld, void* o, float* lse, int B, int S, int nh, int nkv, int d, hipStream_t st);
hipError_t attn_f32_bwd(const void* qkv, int ld, const void* o, const void* dout, const float* lse, float* dvec,
                        void* dqkv, int B, int S, int nh, int nkv, int d, hipStream_t st);

hipError_t gemm(int dtype, const GemmDesc& g, hipStream_t st) {
    return dtype == DT_BF16 ? gemm_bf16(g, st) : gemm_f32(g, st);
}
hipError_t attn_fwd(int dtype, const void* qkv, int ld, void* o, float* lse, int B, int S, int nh, int nkv, int d, hipStream_t st) {
    return dtype == DT_BF16 ? attn_bf16_fwd(qkv, ld, o, lse, B, S, nh, nkv, d, st) : attn_f32_fwd(qkv, ld, o, lse, B, S, nh, nkv, d, st);
}
size_t attn_bwd_scratch_bytes(int dtype, int B, int S, int nh, int nkv, int d) {
    return dtype == DT_BF16 ? attn_bf16_bwd_scratch_bytes(B, S, nh, nkv, d) : 0;
}
hipError_t attn_bwd(int dtype, const void* qkv, int ld, const void* o, const void* dout, const float* lse, float* dvec,
                    void* dqkv, void* scratch, int B, int S, int nh, int nkv, int d,
                    const float* rope_table, int rope_seq, hipStream_t st) {
    // bf16: the kernels take the rotary embedding back out of dq and dk as they write them; fp32: a pass of its own
    if (dtype == DT_BF16) return attn_bf16_bwd(qkv, ld, o, dout, lse, dvec, dqkv, (float*)scratch, B, S, nh, nkv, d, rope_table, rope_seq, st);
    const hipError_t e = attn_f32_bwd(qkv, ld, o, dout, lse, dvec, dqkv, B, S, nh, nkv, d, st);
    if (e != hipSuccess || !rope_table) return e;
    return rope(dtype, dqkv, ld, B * S, S, nh + nkv, d, rope_table, rope_seq, 1, st);
}
}  // namespace hh

using namespace hh;
static_assert(HH_STATIC_SCRATCH_BYTES == STATIC_SCRATCH_BYTES, "the header states the size of the library's scratch array");

// ------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

static int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}
static int hip_fail(hipError_t e, const char* what) {
    return fail(HH_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}
#define HIP_TRY(call)                                        \
    do {                                                     \
        hipError_t e_ = (call);                              \
        if (e_ != hipSuccess) return hip_fail(e_, #call);    \
    } while (0)

extern "C" const char* hh_last_error(void) { return g_err; }
namespace hh {
// for the other translation units of the library
int set_error(int code, const char* msg) { return fail(code, "%s", msg); }
}  // namespace hh

// ------------------------------------------------------------------ context
struct TraceRec {
    hipEvent_t a, b;
    int kind;
    double work;
};
struct hh_ctx {
    int device;
    float* rope_table;  // device: cos[S][d/2] then sin[S][d/2]
    int rope_seq, rope_dim;
    float rope_base;
    std::vector<TraceRec> trace;  // events created by hh_trace_begin
    size_t trace_used;
    bool trace_on;
    uint32_t trace_mask;          // families recorded while trace_on
    void* gemm_ws;                // k-split scratch inside the caller's workspace, set by each hot call
    std::vector<float*> retired_tables;   // rotary tables replaced by a larger one: freed with the context
};

extern "C" int hh_ctx_create(hh_ctx** out, int device) {
    if (!out) return fail(HH_ERR_INVALID_ARG, "hh_ctx_create: out is NULL");
    *out = nullptr;
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess) return hip_fail(e, "hipGetDeviceCount");
    if (device < 0 || device >= n) return fail(HH_ERR_DEVICE, "hh_ctx_create: no HIP device %d (%d visible)", device, n);
    // the library's own scratch array lives at a different address on every GPU: look this GPU's up now
    int prev = 0;
    e = hipGetDevice(&prev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    e = hipSetDevice(device);
    if (e != hipSuccess) return hip_fail(e, "hipSetDevice");
    e = static_scratch_init(device);
    (void)hipSetDevice(prev);
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    hh_ctx* c = new (std::nothrow) hh_ctx{device, nullptr, 0, 0, 0.f, {}, 0, false, 0u, nullptr, {}};
    if (!c) return fail(HH_ERR_INVALID_ARG, "hh_ctx_create: out of host memory");
    *out = c;
    return HH_OK;
}

extern "C" int hh_ctx_destroy(hh_ctx* ctx) {
    if (!ctx) return HH_OK;
    if (ctx->rope_table) (void)hipFree(ctx->rope_table);
    for (float* t : ctx->retired_tables) (void)hipFree(t);
    for (auto& r : ctx->trace) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    delete ctx;
    return HH_OK;
}

// ---------------------------------------------------------------- validation
static int check_cfg(const hh_layer_cfg* c) {
    if (!c) return fail(HH_ERR_INVALID_ARG, "cfg is NULL");
    if (c->dtype != HH_F32 && c->dtype != HH_BF16) return fail(HH_ERR_INVALID_ARG, "cfg.dtype %d is not HH_F32/HH_BF16", c->dtype);
    if (c->hidden <= 0 || c->n_heads <= 0 || c->head_dim <= 0 || c->ffn <= 0 || c->seq <= 0 || c->micro_batch <= 0)
        return fail(HH_ERR_INVALID_ARG, "cfg has a non-positive dimension");
    if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return fail(HH_ERR_INVALID_ARG, "cfg.rms_eps must be >= 0 and rope_base > 0");
    if (c->n_kv_heads <= 0 || c->n_heads % c->n_kv_heads)
        return fail(HH_ERR_UNSUPPORTED_SHAPE, "n_kv_heads (%d) must be positive and divide n_heads (%d)", c->n_kv_heads, c->n_heads);
    if (c->head_dim != 64 && c->head_dim != 128) return fail(HH_ERR_UNSUPPORTED_SHAPE, "head_dim %d: only 64 and 128", c->head_dim);
    const int mult = c->dtype == HH_BF16 ? 64 : 8;
    const long A = (long)c->n_heads * c->head_dim;   // the kv width n_kv_heads*head_dim is a multiple of 64 as well
    if (c->hidden % mult || A % mult || c->ffn % mult)
        return fail(HH_ERR_UNSUPPORTED_SHAPE, "hidden, n_heads*head_dim and ffn must be multiples of %d for this dtype", mult);
    if (c->hidden > 32768) return fail(HH_ERR_UNSUPPORTED_SHAPE, "hidden %d exceeds 32768", c->hidden);
    // The kernels address every buffer with 32-bit byte offsets: outputs below 2^31 bytes, GEMM operands below
    // 2^32 - 2^25.  Packed q|k|v and gate|up gradients that would be larger are written part by part (see the
    // backward), so only the single projections bound the fp32 gradients.
    const long es = c->dtype == HH_BF16 ? 2 : 4;
    const long T = (long)c->seq * c->micro_batch;
    const long Q3 = A + 2L * c->n_kv_heads * c->head_dim;
    const long wide = std::max<long>(std::max<long>(c->hidden, Q3), 2L * c->ffn);
    if (wide > 65535) return fail(HH_ERR_UNSUPPORTED_SHAPE, "a row of %ld elements exceeds 65535", wide);
    if (T * wide * es >= (1L << 31))
        return fail(HH_ERR_UNSUPPORTED_SHAPE, "an activation of %ld x %ld elements reaches 2^31 bytes", T, wide);
    if ((long)c->hidden * std::max<long>(A, c->ffn) * 4 >= (1L << 31))
        return fail(HH_ERR_UNSUPPORTED_SHAPE, "the fp32 gradient of one projection reaches 2^31 bytes");
    if ((long)c->hidden * wide * es >= (1L << 32) - (1L << 25))
        return fail(HH_ERR_UNSUPPORTED_SHAPE, "a packed weight of %d x %ld elements reaches 2^32 bytes", c->hidden, wide);
    return HH_OK;
}

static int check_ptr(const void* p, const char* name) {
    if (!p) return fail(HH_ERR_INVALID_ARG, "%s is NULL", name);
    if ((uintptr_t)p & 15) return fail(HH_ERR_MISALIGNED, "%s is not 16-byte aligned", name);
    return HH_OK;
}
#define TRY(x)                \
    do {                      \
        int rc_ = (x);        \
        if (rc_ != HH_OK) return rc_; \
    } while (0)

static int check_weights(const hh_layer_weights* w) {
    if (!w) return fail(HH_ERR_INVALID_ARG, "weights is NULL");
    TRY(check_ptr(w->g_attn, "weights.g_attn")); TRY(check_ptr(w->wq, "weights.wq")); TRY(check_ptr(w->wk, "weights.wk"));
    TRY(check_ptr(w->wv, "weights.wv")); TRY(check_ptr(w->wo, "weights.wo")); TRY(check_ptr(w->g_mlp, "weights.g_mlp"));
    TRY(check_ptr(w->w_gate, "weights.w_gate")); TRY(check_ptr(w->w_up, "weights.w_up")); TRY(check_ptr(w->w_down, "weights.w_down"));
    return HH_OK;
}
static int check_grads(const hh_layer_grads* g) {
    if (!g) return fail(HH_ERR_INVALID_ARG, "grads is NULL");
    TRY(check_ptr(g->g_attn, "grads.g_attn")); TRY(check_ptr(g->wq, "grads.wq")); TRY(check_ptr(g->wk, "grads.wk"));
    TRY(check_ptr(g->wv, "grads.wv")); TRY(check_ptr(g->wo, "grads.wo")); TRY(check_ptr(g->g_mlp, "grads.g_mlp"));
    TRY(check_ptr(g->w_gate, "grads.w_gate")); TRY(check_ptr(g->w_up, "grads.w_up")); TRY(check_ptr(g->w_down, "grads.w_down"));
    return HH_OK;
}

// ------------------------------------------------------------ buffer layouts
static inline size_t up256(size_t n) { return (n + 255) & ~(size_t)255; }

struct Dims {
    int T, H, A, Akv, Q3, F, S, B, nh, nkv, d, dt;   // Akv = nkv*d; Q3 = A + 2*Akv: width of a q|k|v row
    size_t es;
};
static Dims dims_of(const hh_layer_cfg* c) {
    Dims d;
    d.S = c->seq; d.B = c->micro_batch; d.T = c->seq * c->micro_batch; d.H = c->hidden; d.nh = c->n_heads; d.d = c->head_dim;
    d.A = c->n_heads * c->head_dim; d.nkv = c->n_kv_heads; d.Akv = d.nkv * d.d; d.Q3 = d.A + 2 * d.Akv; d.F = c->ffn; d.dt = c->dtype == HH_BF16 ? DT_BF16 : DT_F32; d.es = dt_size(d.dt);
    return d;
}

struct SavedLayout {
    size_t xn, qkv, a, h, hn, gu, lse, r1, r2, total;
};
static SavedLayout saved_layout(const Dims& d) {
    SavedLayout s;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += up256(bytes); return o; };
    const size_t T = d.T;
    s.xn = take(T * d.H * d.es);
    s.qkv = take(T * d.Q3 * d.es);
    s.a = take(T * d.A * d.es);
    s.h = take(T * d.H * d.es);
    s.hn = take(T * d.H * d.es);
    s.gu = take(T * 2 * d.F * d.es);
    s.lse = take((size_t)d.B * d.nh * d.S * 4);
    s.r1 = take(T * 4);
    s.r2 = take(T * 4);
    s.total = off;
    return s;
}

struct WorkLayout {
    size_t m, dgu, dhn, dh, da, dqkv, dvec, dkv_part, partial, gemm_ws, total;
};
static WorkLayout work_layout(const Dims& d) {
    WorkLayout w;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += up256(bytes); return o; };
    const size_t T = d.T;
    w.m = take(T * d.F * d.es);            // forward: m; backward: dm, then m recomputed in place
    w.dgu = take(T * 2 * d.F * d.es);
    w.dhn = take(T * d.H * d.es);          // d(hn), later d(xn)
    w.dh = take(T * d.H * d.es);
    w.da = take(T * d.A * d.es);
    w.dqkv = take(T * d.Q3 * d.es);
    w.dvec = take((size_t)d.B * d.nh * d.S * 4);
    w.dkv_part = take(attn_bwd_scratch_bytes(d.dt, d.B, d.S, d.nh, d.nkv, d.d));   // partial dK, dV of grouped heads
    w.partial = take((size_t)rmsnorm_bwd_blocks(d.T) * d.H * 4);
    w.gemm_ws = take(d.dt == DT_BF16 ? GEMM_WS_BYTES : 0);
    w.total = off;
    return w;
}

extern "C" int hh_layer_sizes(const hh_layer_cfg* cfg, size_t* saved_bytes, size_t* workspace_bytes) {
    TRY(check_cfg(cfg));
    const Dims d = dims_of(cfg);
    if (saved_bytes) *saved_bytes = saved_layout(d).total;
    if (workspace_bytes) *workspace_bytes = work_layout(d).total;
    return HH_OK;
}

extern "C" int hh_saved_layout_of(const hh_layer_cfg* cfg, hh_saved_layout* out) {
    TRY(check_cfg(cfg));
    if (!out) return fail(HH_ERR_INVALID_ARG, "out is NULL");
    const SavedLayout s = saved_layout(dims_of(cfg));
    out->xn = s.xn; out->qkv = s.qkv; out->a = s.a; out->h = s.h; out->hn = s.hn; out->gate_up = s.gu;
    out->lse = s.lse; out->r1 = s.r1; out->r2 = s.r2; out->total = s.total;
    return HH_OK;
}

static size_t act_bytes(const Dims& d) { return up256((size_t)d.T * d.H * d.es); }

extern "C" int hh_stage_sizes(const hh_layer_cfg* cfg, int n_layers, int n_micro, size_t* saved_pool_bytes,
                              size_t* workspace_bytes) {
    TRY(check_cfg(cfg));
    if (n_layers <= 0 || n_micro <= 0) return fail(HH_ERR_INVALID_ARG, "n_layers and n_micro must be positive");
    const Dims d = dims_of(cfg);
    const size_t per_micro = (size_t)n_layers * saved_layout(d).total + (size_t)(n_layers - 1) * act_bytes(d);
    if (saved_pool_bytes) *saved_pool_bytes = per_micro * (size_t)n_micro;
    if (workspace_bytes) *workspace_bytes = work_layout(d).total + act_bytes(d);  // + the gradient passed between layers
    return HH_OK;
}

extern "C" int hh_layer_flops(const hh_layer_cfg* cfg, double* fwd_flop, double* bwd_flop) {
    TRY(check_cfg(cfg));
    const Dims d = dims_of(cfg);
    const double T = d.T;
    const double gemm = T * (2.0 * (d.Q3 + d.A) * d.H + 6.0 * (double)d.H * d.F);
    const double attn = 4.0 * d.d * d.B * d.nh * ((double)d.S * (d.S + 1) / 2);
    if (fwd_flop) *fwd_flop = gemm + attn;
    if (bwd_flop) *bwd_flop = 2.0 * (gemm + attn);
    return HH_OK;
}

// ------------------------------------------------------------- rotary table
static int ensure_rope(hh_ctx* ctx, const hh_layer_cfg* c) {
    if (ctx->rope_table && ctx->rope_seq >= c->seq && ctx->rope_dim == c->head_dim && ctx->rope_base == c->rope_base) return HH_OK;
    HIP_TRY(hipSetDevice(ctx->device));
    if (ctx->rope_table) {
        // launches already enqueued, and graphs recorded earlier, still read the old table: it stays alive
        // until the context is destroyed
        ctx->retired_tables.push_back(ctx->rope_table);
        ctx->rope_table = nullptr;
    }
    const int S = c->seq, half = c->head_dim / 2;
    std::vector<float> host((size_t)2 * S * half);
    for (int i = 0; i < half; i++) {
        const double theta = std::pow((double)c->rope_base, -2.0 * i / c->head_dim);
        for (int s = 0; s < S; s++) {
            const double phi = s * theta;
            host[(size_t)s * half + i] = (float)std::cos(phi);
            host[(size_t)S * half + (size_t)s * half + i] = (float)std::sin(phi);
        }
    }
    HIP_TRY(hipMalloc((void**)&ctx->rope_table, host.size() * sizeof(float)));
    HIP_TRY(hipMemcpy(ctx->rope_table, host.data(), host.size() * sizeof(float), hipMemcpyHostToDevice));
    ctx->rope_seq = S; ctx->rope_dim = c->head_dim; ctx->rope_base = c->rope_base;
    return HH_OK;
}

extern "C" int hh_ctx_reserve(hh_ctx* ctx, const hh_layer_cfg* cfg) {
    TRY(check_cfg(cfg));
    if (!ctx) return fail(HH_ERR_INVALID_ARG, "ctx is NULL");
    return ensure_rope(ctx, cfg);
}

// ------------------------------------------------------------------ tracing
// When tracing is on, every kernel-family launch is bracketed by two events on the
// launch stream; hh_trace_end turns them into per-family time and work sums.
struct Traced {
    hh_ctx* ctx; hipStream_t st; TraceRec* rec;
    Traced(hh_ctx* c, hipStream_t s, int kind, double work) : ctx(c), st(s), rec(nullptr) {
        if (c->trace_on && ((c->trace_mask >> kind) & 1u) && c->trace_used < c->trace.size()) {
            rec = &c->trace[c->trace_used++];
            rec->kind = kind; rec->work = work;
            (void)hipEventRecord(rec->a, st);
        }
    }
    ~Traced() { if (rec) (void)hipEventRecord(rec->b, st); }
};
#define TR(kind, work, call)                     \
    do {                                         \
        Traced t_(ctx, st, (kind), (double)(work)); \
        HIP_TRY(call);                           \
    } while (0)
static double attn_flop(const Dims& d) { return 4.0 * d.d * d.B * d.nh * ((double)d.S * (d.S + 1) / 2); }
static double gemm_flop(const GemmDesc& g) { return 2.0 * g.M * g.N * g.K; }
static hipError_t tgemm(hh_ctx* ctx, int dt, GemmDesc g, hipStream_t st) {
    Traced t(ctx, st, g.kind, gemm_flop(g));
    g.ws = ctx->gemm_ws; g.ws_bytes = ctx->gemm_ws ? GEMM_WS_BYTES : 0;
    return gemm(dt, g, st);
}

extern "C" int hh_trace_begin(hh_ctx* ctx, int max_launches, uint32_t kind_mask) {
    if (!ctx) return fail(HH_ERR_INVALID_ARG, "ctx is NULL");
    if (max_launches <= 0) return fail(HH_ERR_INVALID_ARG, "max_launches must be positive");
    HIP_TRY(hipSetDevice(ctx->device));
    while ((int)ctx->trace.size() < max_launches) {
        TraceRec r{nullptr, nullptr, 0, 0.0};
        HIP_TRY(hipEventCreate(&r.a));
        hipError_t e = hipEventCreate(&r.b);
        if (e != hipSuccess) { (void)hipEventDestroy(r.a); return hip_fail(e, "hipEventCreate"); }
        ctx->trace.push_back(r);
    }
    ctx->trace_used = 0;
    ctx->trace_mask = kind_mask;
    ctx->trace_on = true;
    return HH_OK;
}

extern "C" int hh_trace_end(hh_ctx* ctx, hh_trace_sum* out, int n_kinds) {
    if (!ctx || !out) return fail(HH_ERR_INVALID_ARG, "ctx or out is NULL");
    if (n_kinds <= 0) return fail(HH_ERR_INVALID_ARG, "n_kinds must be positive");
    ctx->trace_on = false;
    for (int k = 0; k < n_kinds; k++) { out[k].kind = k; out[k].launches = 0; out[k].ms = 0.0; out[k].work = 0.0; }
    for (size_t i = 0; i < ctx->trace_used; i++) {
        const TraceRec& r = ctx->trace[i];
        HIP_TRY(hipEventSynchronize(r.b));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
        if (r.kind < n_kinds) { out[r.kind].launches++; out[r.kind].ms += ms; out[r.kind].work += r.work; }
    }
    ctx->trace_used = 0;
    return HH_OK;
}

// ------------------------------------------------------------ layer forward
static inline char* at(void* base, size_t off) { return (char*)base + off; }
static inline const char* at(const void* base, size_t off) { return (const char*)base + off; }

static GemmDesc desc(int kind, int M, int N, int K, const void* A, int lda, const void* B, int ldb, void* C, int ldc,
                     const void* R = nullptr, int ldr = 0, int out_f32 = 0, int acc = 0) {
    GemmDesc g;
    g.kind = kind; g.M = M; g.N = N; g.K = K; g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
    g.R = R; g.ldr = ldr; g.out_f32 = out_f32; g.accumulate = acc; g.ws = nullptr; g.ws_bytes = 0;
    return g;
}

static int layer_fwd_impl(hh_ctx* ctx, const Dims& d, const hh_layer_cfg* cfg, const hh_layer_weights* w, const void* x,
                          void* y, void* saved, void* ws, hipStream_t st) {
    const SavedLayout sl = saved_layout(d);
    const WorkLayout wl = work_layout(d);
    const int T = d.T, H = d.H, A = d.A, F = d.F, dt = d.dt;
    const size_t es = d.es;
    void* xn = at(saved, sl.xn); void* qkv = at(saved, sl.qkv); void* a = at(saved, sl.a); void* h = at(saved, sl.h);
    void* hn = at(saved, sl.hn); void* gu = at(saved, sl.gu);
    float* lse = (float*)at(saved, sl.lse); float* r1 = (float*)at(saved, sl.r1); float* r2 = (float*)at(saved, sl.r2);
    void* m = at(ws, wl.m);
    ctx->gemm_ws = d.dt == DT_BF16 ? at(ws, wl.gemm_ws) : nullptr;

    TR(HH_TRACE_ELEMENTWISE, 2.0 * T * H * es, rmsnorm_fwd(dt, x, w->g_attn, xn, r1, T, H, cfg->rms_eps, st));
    // q | k | v rows of width A, Akv, Akv (Akv < A with grouped-query attention)
    const int Akv = d.Akv, Q3 = d.Q3;
    const int part_w[3] = {A, Akv, Akv}, part_c[3] = {0, A, A + Akv};
    const bool qkv_packed = (const char*)w->wk == (const char*)w->wq + (size_t)A * H * es &&
                            (const char*)w->wv == (const char*)w->wk + (size_t)Akv * H * es;
    if (qkv_packed) {
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_NT, T, Q3, H, xn, H, w->wq, H, qkv, Q3), st));
    } else {
        const void* ws3[3] = {w->wq, w->wk, w->wv};
        for (int i = 0; i < 3; i++)
            HIP_TRY(tgemm(ctx, dt, desc(GEMM_NT, T, part_w[i], H, xn, H, ws3[i], H, at(qkv, (size_t)part_c[i] * es), Q3), st));
    }
    TR(HH_TRACE_ELEMENTWISE, 2.0 * T * (A + Akv) * es, rope(dt, qkv, Q3, T, d.S, d.nh + d.nkv, d.d, ctx->rope_table, ctx->rope_seq, 0, st));
    TR(HH_TRACE_ATTN_FWD, attn_flop(d), attn_fwd(dt, qkv, Q3, a, lse, d.B, d.S, d.nh, d.nkv, d.d, st));
    HIP_TRY(tgemm(ctx, dt, desc(GEMM_NT, T, H, A, a, A, w->wo, A, h, H, x, H), st));
    TR(HH_TRACE_ELEMENTWISE, 2.0 * T * H * es, rmsnorm_fwd(dt, h, w->g_mlp, hn, r2, T, H, cfg->rms_eps, st));
    const bool gu_packed = (const char*)w->w_up == (const char*)w->w_gate + (size_t)F * H * es;
    if (gu_packed) {
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_NT, T, 2 * F, H, hn, H, w->w_gate, H, gu, 2 * F), st));
    } else {
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_NT, T, F, H, hn, H, w->w_gate, H, gu, 2 * F), st));
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_NT, T, F, H, hn, H, w->w_up, H, at(gu, (size_t)F * es), 2 * F), st));
    }
    TR(HH_TRACE_ELEMENTWISE, 3.0 * T * F * es, swiglu_fwd(dt, gu, m, T, F, st));
    HIP_TRY(tgemm(ctx, dt, desc(GEMM_NT, T, H, F, m, F, w->w_down, F, y, H, h, H), st));
    return HH_OK;
}

extern "C" int hh_layer_fwd(hh_ctx* ctx, const hh_layer_cfg* cfg, const hh_layer_weights* w, const void* x, void* y,
                            void* saved, void* workspace, void* stream) {
    TRY(check_cfg(cfg));
    TRY(check_weights(w));
    TRY(check_ptr(x, "x")); TRY(check_ptr(y, "y")); TRY(check_ptr(workspace, "workspace"));
    if (saved && ((uintptr_t)saved & 15)) return fail(HH_ERR_MISALIGNED, "saved is not 16-byte aligned");
    if (x == y) return fail(HH_ERR_INVALID_ARG, "y must not alias x");
    if (!ctx) return fail(HH_ERR_INVALID_ARG, "ctx is NULL");
    TRY(ensure_rope(ctx, cfg));
    const Dims d = dims_of(cfg);
    void* sv = saved;
    void* wsp = workspace;
    if (!sv) {  // forward only: the saved block lives at the front of the workspace
        sv = workspace;
        wsp = at(workspace, saved_layout(d).total);
    }
    return layer_fwd_impl(ctx, d, cfg, w, x, y, sv, wsp, (hipStream_t)stream);
}

extern "C" int hh_layer_fwd_noalloc(hh_ctx* ctx, const hh_layer_cfg* cfg, const hh_layer_weights* w, const void* x, void* y,
                                    void* stream) {
    TRY(check_cfg(cfg));
    TRY(check_weights(w));
    TRY(check_ptr(x, "x")); TRY(check_ptr(y, "y"));
    if (x == y) return fail(HH_ERR_INVALID_ARG, "y must not alias x");
    if (!ctx) return fail(HH_ERR_INVALID_ARG, "ctx is NULL");
    // the rotary table is the one thing the ordinary forward may allocate: here it has to be there already
    if (!(ctx->rope_table && ctx->rope_seq >= cfg->seq && ctx->rope_dim == cfg->head_dim && ctx->rope_base == cfg->rope_base))
        return fail(HH_ERR_INVALID_ARG, "hh_layer_fwd_noalloc: no rotary table for this (seq, head_dim, rope_base): call hh_ctx_reserve first");
    const Dims d = dims_of(cfg);
    const size_t saved_b = saved_layout(d).total, need = saved_b + work_layout(d).total;
    if (need > STATIC_SCRATCH_BYTES)
        return fail(HH_ERR_BUFFER_TOO_SMALL, "hh_layer_fwd_noalloc: this shape needs %zu bytes of scratch, the library's array holds %zu",
                    need, (size_t)STATIC_SCRATCH_BYTES);
    void* base = static_scratch(ctx->device);
    if (!base) return fail(HH_ERR_DEVICE, "hh_layer_fwd_noalloc: the scratch array of device %d was never looked up", ctx->device);
    // same carving as hh_layer_fwd with saved == NULL: the saved block first, the workspace behind it
    return layer_fwd_impl(ctx, d, cfg, w, x, y, base, at(base, saved_b), (hipStream_t)stream);
}

// ----------------------------------------------------------- layer backward
static int layer_bwd_impl(hh_ctx* ctx, const Dims& d, const hh_layer_cfg* cfg, const hh_layer_weights* w, const void* x,
                          const void* saved, const void* dy, void* dx, const hh_layer_grads* g, int acc, void* ws,
                          hipStream_t st) {
    (void)cfg;
    const SavedLayout sl = saved_layout(d);
    const WorkLayout wl = work_layout(d);
    const int T = d.T, H = d.H, A = d.A, F = d.F, dt = d.dt;
    const size_t es = d.es;
    const void* xn = at(saved, sl.xn); const void* qkv = at(saved, sl.qkv); const void* a = at(saved, sl.a);
    const void* h = at(saved, sl.h); const void* hn = at(saved, sl.hn); const void* gu = at(saved, sl.gu);
    const float* lse = (const float*)at(saved, sl.lse);
    const float* r1 = (const float*)at(saved, sl.r1); const float* r2 = (const float*)at(saved, sl.r2);
    void* m = at(ws, wl.m); void* dgu = at(ws, wl.dgu); void* dhn = at(ws, wl.dhn); void* dh = at(ws, wl.dh);
    void* da = at(ws, wl.da); void* dqkv = at(ws, wl.dqkv);
    float* dvec = (float*)at(ws, wl.dvec); float* partial = (float*)at(ws, wl.partial);
    const int nblk = rmsnorm_bwd_blocks(T);
    acc = acc ? 1 : 0;
    ctx->gemm_ws = d.dt == DT_BF16 ? at(ws, wl.gemm_ws) : nullptr;

    // MLP branch: y = h + m Wd^T
    HIP_TRY(tgemm(ctx, dt, desc(GEMM_NN, T, F, H, dy, H, w->w_down, F, m, F), st));                 // dm (in the m buffer)
    TR(HH_TRACE_ELEMENTWISE, 6.0 * T * F * es, swiglu_bwd(dt, m, gu, dgu, m, T, F, st));                                          // dgate|dup, m
    HIP_TRY(tgemm(ctx, dt, desc(GEMM_TN, H, F, T, dy, H, m, F, g->w_down, F, nullptr, 0, 1, acc), st));
    const bool gu_packed = (const char*)w->w_up == (const char*)w->w_gate + (size_t)F * H * es;
    const bool dgu_packed = (char*)g->w_up == (char*)g->w_gate + (size_t)F * H * 4 && (size_t)2 * F * H * 4 < ((size_t)1 << 31);
    if (dgu_packed) {
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_TN, 2 * F, H, T, dgu, 2 * F, hn, H, g->w_gate, H, nullptr, 0, 1, acc), st));
    } else {
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_TN, F, H, T, dgu, 2 * F, hn, H, g->w_gate, H, nullptr, 0, 1, acc), st));
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_TN, F, H, T, at(dgu, (size_t)F * es), 2 * F, hn, H, g->w_up, H, nullptr, 0, 1, acc), st));
    }
    if (gu_packed) {
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_NN, T, H, 2 * F, dgu, 2 * F, w->w_gate, H, dhn, H), st));
    } else {
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_NN, T, H, F, dgu, 2 * F, w->w_gate, H, dhn, H), st));
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_NN, T, H, F, at(dgu, (size_t)F * es), 2 * F, w->w_up, H, dhn, H, dhn, H), st));
    }
    TR(HH_TRACE_ELEMENTWISE, 4.0 * T * H * es, rmsnorm_bwd(dt, dhn, h, r2, w->g_mlp, dy, dh, partial, T, H, st));                // dh = dy + norm-bwd
    TR(HH_TRACE_ELEMENTWISE, 4.0 * nblk * H, colsum_reduce(partial, nblk, H, g->g_mlp, acc, st));

    // attention branch: h = x + a Wo^T
    HIP_TRY(tgemm(ctx, dt, desc(GEMM_TN, H, A, T, dh, H, a, A, g->wo, A, nullptr, 0, 1, acc), st));
    HIP_TRY(tgemm(ctx, dt, desc(GEMM_NN, T, A, H, dh, H, w->wo, A, da, A), st));
    const int Akv = d.Akv, Q3 = d.Q3;
    const int part_w[3] = {A, Akv, Akv}, part_c[3] = {0, A, A + Akv};
    // dq | dk | dv of the rotated q, k and of v, with the rotary embedding taken back out of dq and dk
    TR(HH_TRACE_ATTN_BWD, 2.0 * attn_flop(d), attn_bwd(dt, qkv, Q3, a, da, lse, dvec, dqkv, at(ws, wl.dkv_part), d.B, d.S, d.nh, d.nkv, d.d,
                                                       ctx->rope_table, ctx->rope_seq, st));
    const bool qkv_packed = (const char*)w->wk == (const char*)w->wq + (size_t)A * H * es &&
                            (const char*)w->wv == (const char*)w->wk + (size_t)Akv * H * es;
    const bool dqkv_packed = (char*)g->wk == (char*)g->wq + (size_t)A * H * 4 && (char*)g->wv == (char*)g->wk + (size_t)Akv * H * 4 &&
                             (size_t)Q3 * H * 4 < ((size_t)1 << 31);
    if (dqkv_packed) {
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_TN, Q3, H, T, dqkv, Q3, xn, H, g->wq, H, nullptr, 0, 1, acc), st));
    } else {
        float* gs[3] = {g->wq, g->wk, g->wv};
        for (int i = 0; i < 3; i++)
            HIP_TRY(tgemm(ctx, dt, desc(GEMM_TN, part_w[i], H, T, at(dqkv, (size_t)part_c[i] * es), Q3, xn, H, gs[i], H, nullptr, 0, 1, acc), st));
    }
    void* dxn = dhn;
    if (qkv_packed) {
        HIP_TRY(tgemm(ctx, dt, desc(GEMM_NN, T, H, Q3, dqkv, Q3, w->wq, H, dxn, H), st));
    } else {
        const void* ws3[3] = {w->wq, w->wk, w->wv};
        for (int i = 0; i < 3; i++)
            HIP_TRY(tgemm(ctx, dt, desc(GEMM_NN, T, H, part_w[i], at(dqkv, (size_t)part_c[i] * es), Q3, ws3[i], H, dxn, H,
                                  i ? dxn : nullptr, H), st));
    }
    TR(HH_TRACE_ELEMENTWISE, 4.0 * T * H * es, rmsnorm_bwd(dt, dxn, x, r1, w->g_attn, dh, dx, partial, T, H, st));              // dx = dh + norm-bwd
    TR(HH_TRACE_ELEMENTWISE, 4.0 * nblk * H, colsum_reduce(partial, nblk, H, g->g_attn, acc, st));
    return HH_OK;
}

extern "C" int hh_layer_bwd(hh_ctx* ctx, const hh_layer_cfg* cfg, const hh_layer_weights* w, const void* x,
                            const void* saved, const void* dy, void* dx, const hh_layer_grads* grads, int accumulate,
                            void* workspace, void* stream) {
    TRY(check_cfg(cfg));
    TRY(check_weights(w));
    TRY(check_grads(grads));
    TRY(check_ptr(x, "x")); TRY(check_ptr(saved, "saved")); TRY(check_ptr(dy, "dy")); TRY(check_ptr(dx, "dx"));
    TRY(check_ptr(workspace, "workspace"));
    if (!ctx) return fail(HH_ERR_INVALID_ARG, "ctx is NULL");
    TRY(ensure_rope(ctx, cfg));
    const Dims d = dims_of(cfg);
    return layer_bwd_impl(ctx, d, cfg, w, x, saved, dy, dx, grads, accumulate, workspace, (hipStream_t)stream);
}

// --------------------------------------------------------------- stage step
struct StagePool {
    size_t saved_sz, act_sz, per_micro;
    char* base;
    int k;
    void* saved(int m, int l) const { return base + (size_t)m * per_micro + (size_t)l * (saved_sz + act_sz); }
    // output of layer l (< k-1) = input of layer l+1
    void* act(int m, int l) const { return base + (size_t)m * per_micro + (size_t)l * (saved_sz + act_sz) + saved_sz; }
};
static StagePool stage_pool(const Dims& d, int k, void* pool) {
    StagePool p;
    p.saved_sz = saved_layout(d).total; p.act_sz = act_bytes(d); p.k = k;
    p.per_micro = (size_t)k * p.saved_sz + (size_t)(k - 1) * p.act_sz;
    p.base = (char*)pool;
    return p;
}

static int check_stage_args(const hh_layer_cfg* cfg, int n_layers, const hh_layer_weights* w, const hh_layer_grads* g) {
    TRY(check_cfg(cfg));
    if (n_layers <= 0) return fail(HH_ERR_INVALID_ARG, "n_layers must be positive");
    if (!w || !g) return fail(HH_ERR_INVALID_ARG, "weights / grads array is NULL");
    for (int l = 0; l < n_layers; l++) {
        TRY(check_weights(&w[l]));
        TRY(check_grads(&g[l]));
    }
    return HH_OK;
}

// Forward of micro-batch m through the stage, activations into pool slot `slot`.
static int stage_fwd(hh_ctx* ctx, const Dims& d, const hh_layer_cfg* cfg, int k, const hh_layer_weights* w, const StagePool& p,
                     int slot, const void* x, void* y, void* workspace, hipStream_t st) {
    for (int l = 0; l < k; l++) {
        const void* in = l == 0 ? x : p.act(slot, l - 1);
        void* out = l == k - 1 ? y : p.act(slot, l);
        TRY(layer_fwd_impl(ctx, d, cfg, &w[l], in, out, p.saved(slot, l), workspace, st));
    }
    return HH_OK;
}
// Backward of the micro-batch whose activations sit in pool slot `slot`.
static int stage_bwd(hh_ctx* ctx, const Dims& d, const hh_layer_cfg* cfg, int k, const hh_layer_weights* w, const hh_layer_grads* g,
                     const StagePool& p, int slot, const void* x, const void* dy, void* dx, int acc, void* workspace, hipStream_t st) {
    void* gbuf = at(workspace, work_layout(d).total);  // gradient flowing between layers, updated in place
    for (int l = k - 1; l >= 0; l--) {
        const void* in = l == 0 ? x : p.act(slot, l - 1);
        const void* gin = l == k - 1 ? dy : gbuf;
        void* gout = l == 0 ? dx : gbuf;
        TRY(layer_bwd_impl(ctx, d, cfg, &w[l], in, p.saved(slot, l), gin, gout, &g[l], acc, workspace, st));
    }
    return HH_OK;
}

// Both schedules: forward of the first n_live micro-batches, then backward of m followed by forward of
// m + n_live.  n_live == n_micro is "all forwards, then all backwards".  Backward always visits the
// micro-batches in ascending order, so the fp32 sums are formed in the same order for every n_live.
static int stage_run(hh_ctx* ctx, const hh_layer_cfg* cfg, int n_layers, const hh_layer_weights* w, int n_micro, int n_live,
                     const void* const* x, void* const* y, const void* const* dy, void* const* dx, const hh_layer_grads* g,
                     int zero_grads_first, void* saved_pool, void* workspace, void* stream) {
    TRY(check_stage_args(cfg, n_layers, w, g));
    if (n_micro <= 0) return fail(HH_ERR_INVALID_ARG, "n_micro must be positive");
    if (n_live <= 0 || n_live > n_micro) return fail(HH_ERR_INVALID_ARG, "n_live must be in 1..n_micro (got %d, n_micro %d)", n_live, n_micro);
    if (!x || !y || !dy || !dx) return fail(HH_ERR_INVALID_ARG, "x / y / dy / dx pointer array is NULL");
    for (int m = 0; m < n_micro; m++) {
        TRY(check_ptr(x[m], "x[m]")); TRY(check_ptr(y[m], "y[m]")); TRY(check_ptr(dy[m], "dy[m]")); TRY(check_ptr(dx[m], "dx[m]"));
        if (x[m] == y[m]) return fail(HH_ERR_INVALID_ARG, "y[m] must not alias x[m]");
    }
    TRY(check_ptr(saved_pool, "saved_pool")); TRY(check_ptr(workspace, "workspace"));
    if (!ctx) return fail(HH_ERR_INVALID_ARG, "ctx is NULL");
    TRY(ensure_rope(ctx, cfg));
    const Dims d = dims_of(cfg);
    const StagePool p = stage_pool(d, n_layers, saved_pool);
    hipStream_t st = (hipStream_t)stream;
    for (int m = 0; m < n_live; m++) TRY(stage_fwd(ctx, d, cfg, n_layers, w, p, m, x[m], y[m], workspace, st));
    for (int m = 0; m < n_micro; m++) {
        const int acc = (m > 0 || !zero_grads_first) ? 1 : 0;
        const int slot = m % n_live;
        TRY(stage_bwd(ctx, d, cfg, n_layers, w, g, p, slot, x[m], dy[m], dx[m], acc, workspace, st));
        const int nxt = m + n_live;   // its activations take the slot just released
        if (nxt < n_micro) TRY(stage_fwd(ctx, d, cfg, n_layers, w, p, slot, x[nxt], y[nxt], workspace, st));
    }
    return HH_OK;
}

extern "C" int hh_stage_step(hh_ctx* ctx, const hh_layer_cfg* cfg, int n_layers, const hh_layer_weights* w, int n_micro,
                             const void* const* x, void* const* y, const void* const* dy, void* const* dx,
                             const hh_layer_grads* g, int zero_grads_first, void* saved_pool, void* workspace, void* stream) {
    return stage_run(ctx, cfg, n_layers, w, n_micro, n_micro, x, y, dy, dx, g, zero_grads_first, saved_pool, workspace, stream);
}

extern "C" int hh_stage_step_1f1b(hh_ctx* ctx, const hh_layer_cfg* cfg, int n_layers, const hh_layer_weights* w, int n_micro,
                                  int n_live, const void* const* x, void* const* y, const void* const* dy, void* const* dx,
                                  const hh_layer_grads* g, int zero_grads_first, void* saved_pool, void* workspace,
                                  void* stream) {
    return stage_run(ctx, cfg, n_layers, w, n_micro, n_live, x, y, dy, dx, g, zero_grads_first, saved_pool, workspace, stream);
}

// ------------------------------------------------------------------ profile
static float median(std::vector<float>& v) {
    std::sort(v.begin(), v.end());
    const size_t n = v.size();
    return n % 2 ? v[n / 2] : 0.5f * (v[n / 2 - 1] + v[n / 2]);
}

extern "C" int hh_layer_profile(hh_ctx* ctx, const hh_layer_cfg* cfg, int n_layers, const hh_layer_weights* w,
                                const hh_layer_grads* g, const void* x, const void* dy, int warmup, int iters,
                                void* saved_pool, void* workspace, hh_profile_rec* out, void* stream) {
    TRY(check_stage_args(cfg, n_layers, w, g));
    if (warmup < 0 || iters <= 0) return fail(HH_ERR_INVALID_ARG, "warmup must be >= 0 and iters > 0");
    TRY(check_ptr(x, "x")); TRY(check_ptr(dy, "dy")); TRY(check_ptr(saved_pool, "saved_pool")); TRY(check_ptr(workspace, "workspace"));
    if (!out) return fail(HH_ERR_INVALID_ARG, "out is NULL");
    if (!ctx) return fail(HH_ERR_INVALID_ARG, "ctx is NULL");
    TRY(ensure_rope(ctx, cfg));
    const Dims d = dims_of(cfg);
    const StagePool p = stage_pool(d, n_layers, saved_pool);
    hipStream_t st = (hipStream_t)stream;
    void* gbuf = at(workspace, work_layout(d).total);
    // the last layer's output has no slot in the pool (the caller's y in a stage step): park it in gbuf,
    // which is free during the forward sweep
    const int k = n_layers;
    std::vector<hipEvent_t> ev((size_t)4 * k);
    for (auto& e : ev) e = nullptr;
    int rc = HH_OK;
    auto cleanup = [&]() { for (auto e : ev) if (e) (void)hipEventDestroy(e); };
    for (auto& e : ev) {
        hipError_t he = hipEventCreate(&e);
        if (he != hipSuccess) { cleanup(); return hip_fail(he, "hipEventCreate"); }
    }
    std::vector<std::vector<float>> tf(k), tb(k);
    for (int it = 0; it < warmup + iters && rc == HH_OK; it++) {
        for (int l = 0; l < k && rc == HH_OK; l++) {
            const void* in = l == 0 ? x : p.act(0, l - 1);
            void* o = l == k - 1 ? gbuf : p.act(0, l);
            (void)hipEventRecord(ev[4 * l], st);
            rc = layer_fwd_impl(ctx, d, cfg, &w[l], in, o, p.saved(0, l), workspace, st);
            (void)hipEventRecord(ev[4 * l + 1], st);
        }
        for (int l = k - 1; l >= 0 && rc == HH_OK; l--) {
            const void* in = l == 0 ? x : p.act(0, l - 1);
            const void* gin = l == k - 1 ? dy : gbuf;
            (void)hipEventRecord(ev[4 * l + 2], st);
            rc = layer_bwd_impl(ctx, d, cfg, &w[l], in, p.saved(0, l), gin, gbuf, &g[l], 1, workspace, st);
            (void)hipEventRecord(ev[4 * l + 3], st);
        }
        if (rc != HH_OK) break;
        hipError_t he = hipStreamSynchronize(st);
        if (he != hipSuccess) { rc = hip_fail(he, "hipStreamSynchronize"); break; }
        if (it >= warmup)
            for (int l = 0; l < k; l++) {
                float a = 0.f, b = 0.f;
                (void)hipEventElapsedTime(&a, ev[4 * l], ev[4 * l + 1]);
                (void)hipEventElapsedTime(&b, ev[4 * l + 2], ev[4 * l + 3]);
                tf[l].push_back(a);
                tb[l].push_back(b);
            }
    }
    cleanup();
    if (rc != HH_OK) return rc;
    double ff = 0, bf = 0;
    (void)hh_layer_flops(cfg, &ff, &bf);
    const size_t A = d.A;
    const uint64_t nparam = 2ull * d.H + (2ull * A + 2ull * d.Akv) * d.H + 3ull * (uint64_t)d.F * d.H;
    for (int l = 0; l < k; l++) {
        hh_profile_rec& r = out[l];
        r.layer = l;
        r.fwd_ms = median(tf[l]);
        r.bwd_ms = median(tb[l]);
        r.fwd_flop = ff; r.bwd_flop = bf;
        r.fwd_tflops = (float)(ff / (r.fwd_ms * 1e-3) * 1e-12);
        r.bwd_tflops = (float)(bf / (r.bwd_ms * 1e-3) * 1e-12);
        r.weight_bytes = nparam * d.es;
        r.grad_bytes = nparam * 4;
        r.saved_act_bytes = p.saved_sz + (uint64_t)d.T * d.H * d.es;  // the saved block plus the layer's input
        r.p2p_bytes = (uint64_t)d.B * d.S * d.H * 2;
        r.workspace_bytes = work_layout(d).total + act_bytes(d);
    }
    return HH_OK;
}
