"""ctypes binding of libhh.so: the same entry points as include/hh.h, argument marshalling only.

Every numeric step runs in the library's HIP kernels.  PyTorch tensors are used
as owners of device memory (``tensor.data_ptr()``) and for the current stream;
there is no fallback path: if the library is missing, importing fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Sequence

# PyTorch-ROCm ships its own HIP runtime.  It has to be in the process before libhh.so is
# opened so that the library binds to that same runtime (one runtime per process: streams
# and device pointers are shared with torch).
import torch  # noqa: F401

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhh.so")

HH_OK = 0
HH_ERR_INVALID_ARG = -1
HH_ERR_UNSUPPORTED_SHAPE = -2
HH_ERR_BUFFER_TOO_SMALL = -3
HH_ERR_MISALIGNED = -4
HH_ERR_DEVICE = -5
HH_F32 = 0
HH_BF16 = 1
HH_STATIC_SCRATCH_BYTES = 128 << 20

WEIGHT_FIELDS = ("g_attn", "wq", "wk", "wv", "wo", "g_mlp", "w_gate", "w_up", "w_down")
EXPORTS = ("hh_last_error", "hh_ctx_create", "hh_ctx_destroy", "hh_ctx_reserve", "hh_layer_flops", "hh_layer_sizes",
           "hh_saved_layout_of", "hh_layer_fwd", "hh_layer_fwd_noalloc", "hh_layer_bwd", "hh_stage_sizes", "hh_stage_step", "hh_stage_step_1f1b", "hh_layer_profile", "hh_trace_begin",
           "hh_trace_end", "hh_sim_pipeline", "hh_sim_weighted_mean", "hh_plan_layers", "hh_plan_order", "hh_plan_cluster")
TRACE_KINDS = ("gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd", "attn_bwd", "elementwise")


class hh_layer_cfg(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn", C.c_int32), ("seq", C.c_int32), ("micro_batch", C.c_int32), ("rms_eps", C.c_float),
                ("rope_base", C.c_float), ("dtype", C.c_int32)]


class hh_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class hh_layer_grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class hh_profile_rec(C.Structure):
    _fields_ = [("layer", C.c_int32), ("fwd_ms", C.c_float), ("bwd_ms", C.c_float), ("fwd_flop", C.c_double),
                ("bwd_flop", C.c_double), ("fwd_tflops", C.c_float), ("bwd_tflops", C.c_float),
                ("weight_bytes", C.c_uint64), ("grad_bytes", C.c_uint64), ("saved_act_bytes", C.c_uint64),
                ("p2p_bytes", C.c_uint64),
                ("workspace_bytes", C.c_uint64)]


class hh_saved_layout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("xn", "qkv", "a", "h", "hn", "gate_up", "lse", "r1", "r2", "total")]


class hh_trace_sum(C.Structure):
    _fields_ = [("kind", C.c_int32), ("launches", C.c_int32), ("ms", C.c_double), ("work", C.c_double)]


class hh_sim_stage(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_devices", C.c_int32), ("fwd_ms", C.c_double), ("bwd_ms", C.c_double),
                ("peak_tflops", C.c_double), ("link_gbytes_per_s", C.c_double), ("weight_bytes", C.c_uint64),
                ("grad_bytes", C.c_uint64), ("optimizer_bytes", C.c_uint64), ("saved_act_bytes", C.c_uint64),
                ("memory_bytes", C.c_uint64)]


class hh_sim_result(C.Structure):
    _fields_ = [("iter_ms", C.c_double), ("bubble_fraction", C.c_double), ("tokens_per_s_per_device", C.c_double),
                ("tflops_per_device", C.c_double), ("mean_peak_tflops", C.c_double), ("mfu", C.c_double),
                ("n_devices", C.c_int64), ("search_truncated", C.c_int32), ("reserved_", C.c_int32)]


class hh_cluster_group(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("devices_per_node", C.c_int32), ("fwd_ms_tp", C.c_double * 4), ("bwd_ms_tp", C.c_double * 4),
                ("saved_act_bytes_tp", C.c_uint64 * 4), ("peak_tflops", C.c_double), ("link_gbytes_per_s", C.c_double),
                ("dp_gbytes_per_s", C.c_double), ("weight_bytes", C.c_uint64), ("grad_bytes", C.c_uint64),
                ("optimizer_bytes", C.c_uint64), ("memory_bytes", C.c_uint64)]


class hh_cluster_plan(C.Structure):
    _fields_ = [("data_parallel", C.c_int32), ("tensor_parallel", C.c_int32 * 8), ("stages", C.c_int32 * 8), ("order", C.c_int32 * 8),
                ("n_stages", C.c_int32), ("n_micro", C.c_int32), ("strategies_costed", C.c_int32), ("pipeline_ms", C.c_double),
                ("grad_allreduce_ms", C.c_double), ("sim", hh_sim_result)]


class HHError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("hh error %d: %s" % (code, msg))
        self.code = code


def _load() -> C.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError("%s is missing: build it with `python -m paper_2405_16256_amd.build` "
                          "(there is no fallback path)" % _LIB_PATH)
    lib = C.CDLL(_LIB_PATH)
    vp, i, sz = C.c_void_p, C.c_int, C.POINTER(C.c_size_t)
    cfgp, wp, gp = C.POINTER(hh_layer_cfg), C.POINTER(hh_layer_weights), C.POINTER(hh_layer_grads)
    lib.hh_last_error.restype = C.c_char_p
    lib.hh_last_error.argtypes = []
    sigs = {
        "hh_ctx_create": [C.POINTER(vp), i],
        "hh_ctx_destroy": [vp],
        "hh_ctx_reserve": [vp, cfgp],
        "hh_layer_flops": [cfgp, C.POINTER(C.c_double), C.POINTER(C.c_double)],
        "hh_layer_sizes": [cfgp, sz, sz],
        "hh_saved_layout_of": [cfgp, C.POINTER(hh_saved_layout)],
        "hh_layer_fwd": [vp, cfgp, wp, vp, vp, vp, vp, vp],
        "hh_layer_fwd_noalloc": [vp, cfgp, wp, vp, vp, vp],
        "hh_layer_bwd": [vp, cfgp, wp, vp, vp, vp, vp, gp, i, vp, vp],
        "hh_stage_sizes": [cfgp, i, i, sz, sz],
        "hh_stage_step": [vp, cfgp, i, wp, i, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), gp, i, vp, vp, vp],
        "hh_stage_step_1f1b": [vp, cfgp, i, wp, i, i, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), gp, i, vp, vp,
                               vp],
        "hh_layer_profile": [vp, cfgp, i, wp, gp, vp, vp, i, i, vp, vp, C.POINTER(hh_profile_rec), vp],
        "hh_trace_begin": [vp, i, C.c_uint32],
        "hh_trace_end": [vp, C.POINTER(hh_trace_sum), i],
        "hh_sim_pipeline": [C.POINTER(hh_sim_stage), i, i, i, i, i, i, C.c_double, C.POINTER(hh_sim_result), C.POINTER(C.c_double),
                            C.POINTER(C.c_uint64)],
        "hh_sim_weighted_mean": [C.POINTER(C.c_double), C.POINTER(C.c_int64), i, C.POINTER(C.c_double)],
        "hh_plan_layers": [C.POINTER(hh_sim_stage), i, i, i, i, i, i, i, C.c_double, i, C.POINTER(C.c_int32),
                           C.POINTER(hh_sim_result)],
        "hh_plan_order": [C.POINTER(hh_sim_stage), C.POINTER(C.c_int32), i, C.c_double, i, i, i, i, i, i, C.c_double, i,
                          C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(hh_sim_result)],
        "hh_plan_cluster": [C.POINTER(hh_cluster_group), i, C.c_double, i, i, i, i, i, C.c_double, i, C.POINTER(hh_cluster_plan),
                            C.POINTER(C.c_int32), i],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name)
        fn.restype = C.c_int
        fn.argtypes = args
    return lib


lib = _load()


def hh_last_error() -> str:
    return lib.hh_last_error().decode()


def _check(rc: int) -> None:
    if rc != HH_OK:
        raise HHError(rc, hh_last_error())


def _ptr(t) -> int | None:
    """Device address of a torch tensor, or an int / None passed through."""
    if t is None or isinstance(t, int):
        return t
    return t.data_ptr()


def make_cfg(hidden, n_heads, head_dim, ffn, seq, micro_batch=1, rms_eps=1e-5, rope_base=10000.0, dtype=HH_BF16,
             n_kv_heads=None) -> hh_layer_cfg:
    return hh_layer_cfg(hidden, n_heads, n_heads if n_kv_heads is None else n_kv_heads, head_dim, ffn, seq,
                        micro_batch, rms_eps, rope_base, dtype)


def make_weights(w: dict) -> hh_layer_weights:
    return hh_layer_weights(*[_ptr(w[n]) for n in WEIGHT_FIELDS])


def make_grads(g: dict) -> hh_layer_grads:
    return hh_layer_grads(*[_ptr(g[n]) for n in WEIGHT_FIELDS])


def hh_ctx_create(device: int = 0) -> int:
    out = C.c_void_p()
    _check(lib.hh_ctx_create(C.byref(out), device))
    return out.value


def hh_ctx_destroy(ctx: int) -> None:
    _check(lib.hh_ctx_destroy(ctx))


def hh_ctx_reserve(ctx: int, cfg: hh_layer_cfg) -> None:
    _check(lib.hh_ctx_reserve(ctx, C.byref(cfg)))


def hh_layer_flops(cfg: hh_layer_cfg) -> tuple[float, float]:
    f, b = C.c_double(), C.c_double()
    _check(lib.hh_layer_flops(C.byref(cfg), C.byref(f), C.byref(b)))
    return f.value, b.value


def hh_layer_sizes(cfg: hh_layer_cfg) -> tuple[int, int]:
    s, w = C.c_size_t(), C.c_size_t()
    _check(lib.hh_layer_sizes(C.byref(cfg), C.byref(s), C.byref(w)))
    return s.value, w.value


def hh_saved_layout_of(cfg: hh_layer_cfg) -> hh_saved_layout:
    out = hh_saved_layout()
    _check(lib.hh_saved_layout_of(C.byref(cfg), C.byref(out)))
    return out


def hh_stage_sizes(cfg: hh_layer_cfg, n_layers: int, n_micro: int) -> tuple[int, int]:
    s, w = C.c_size_t(), C.c_size_t()
    _check(lib.hh_stage_sizes(C.byref(cfg), n_layers, n_micro, C.byref(s), C.byref(w)))
    return s.value, w.value


def hh_layer_fwd(ctx, cfg, weights: hh_layer_weights, x, y, saved, workspace, stream=0) -> None:
    _check(lib.hh_layer_fwd(ctx, C.byref(cfg), C.byref(weights), _ptr(x), _ptr(y), _ptr(saved), _ptr(workspace), stream))


def hh_layer_fwd_noalloc(ctx, cfg, weights: hh_layer_weights, x, y, stream=0) -> None:
    _check(lib.hh_layer_fwd_noalloc(ctx, C.byref(cfg), C.byref(weights), _ptr(x), _ptr(y), stream))


def hh_layer_bwd(ctx, cfg, weights: hh_layer_weights, x, saved, dy, dx, grads: hh_layer_grads, accumulate, workspace,
                 stream=0) -> None:
    _check(lib.hh_layer_bwd(ctx, C.byref(cfg), C.byref(weights), _ptr(x), _ptr(saved), _ptr(dy), _ptr(dx),
                            C.byref(grads), int(accumulate), _ptr(workspace), stream))


def _ptr_array(ts: Sequence):
    return (C.c_void_p * len(ts))(*[_ptr(t) for t in ts])


def hh_stage_step(ctx, cfg, weights: Sequence[hh_layer_weights], x: Sequence, y: Sequence, dy: Sequence, dx: Sequence,
                  grads: Sequence[hh_layer_grads], zero_grads_first, saved_pool, workspace, stream=0) -> None:
    k, m = len(weights), len(x)
    assert len(grads) == k and len(y) == m and len(dy) == m and len(dx) == m
    warr = (hh_layer_weights * k)(*weights)
    garr = (hh_layer_grads * k)(*grads)
    _check(lib.hh_stage_step(ctx, C.byref(cfg), k, warr, m, _ptr_array(x), _ptr_array(y), _ptr_array(dy), _ptr_array(dx),
                             garr, int(zero_grads_first), _ptr(saved_pool), _ptr(workspace), stream))


def hh_stage_step_1f1b(ctx, cfg, weights: Sequence[hh_layer_weights], n_live: int, x: Sequence, y: Sequence, dy: Sequence,
                       dx: Sequence, grads: Sequence[hh_layer_grads], zero_grads_first, saved_pool, workspace, stream=0) -> None:
    k, m = len(weights), len(x)
    assert len(grads) == k and len(y) == m and len(dy) == m and len(dx) == m
    warr = (hh_layer_weights * k)(*weights)
    garr = (hh_layer_grads * k)(*grads)
    _check(lib.hh_stage_step_1f1b(ctx, C.byref(cfg), k, warr, m, int(n_live), _ptr_array(x), _ptr_array(y), _ptr_array(dy),
                                  _ptr_array(dx), garr, int(zero_grads_first), _ptr(saved_pool), _ptr(workspace), stream))


def hh_layer_profile(ctx, cfg, weights: Sequence[hh_layer_weights], grads: Sequence[hh_layer_grads], x, dy, warmup, iters,
                     saved_pool, workspace, stream=0) -> list[hh_profile_rec]:
    k = len(weights)
    warr = (hh_layer_weights * k)(*weights)
    garr = (hh_layer_grads * k)(*grads)
    out = (hh_profile_rec * k)()
    _check(lib.hh_layer_profile(ctx, C.byref(cfg), k, warr, garr, _ptr(x), _ptr(dy), warmup, iters, _ptr(saved_pool),
                                _ptr(workspace), out, stream))
    return list(out)


def hh_trace_begin(ctx, max_launches: int, kinds=None) -> None:
    """kinds: family names from TRACE_KINDS to record (None: all)."""
    mask = 0xFFFFFFFF if kinds is None else sum(1 << TRACE_KINDS.index(k) for k in kinds)
    _check(lib.hh_trace_begin(ctx, max_launches, mask))


def hh_trace_end(ctx) -> dict:
    """{family: (launches, total_ms, total_work)} for the launches since hh_trace_begin."""
    out = (hh_trace_sum * len(TRACE_KINDS))()
    _check(lib.hh_trace_end(ctx, out, len(TRACE_KINDS)))
    return {TRACE_KINDS[r.kind]: (r.launches, r.ms, r.work) for r in out}


# ---------------------------------------------------------------- predictor (host only)
def hh_sim_pipeline(stages: Sequence[hh_sim_stage], n_micro, micro_batch, seq, hidden, data_parallel, flop_per_layer):
    """-> (hh_sim_result, finish_ms per stage, peak bytes per stage)"""
    n = len(stages)
    arr = (hh_sim_stage * max(n, 1))(*stages)
    res = hh_sim_result()
    fin = (C.c_double * max(n, 1))()
    peak = (C.c_uint64 * max(n, 1))()
    _check(lib.hh_sim_pipeline(arr, n, n_micro, micro_batch, seq, hidden, data_parallel, float(flop_per_layer), C.byref(res), fin,
                               peak))
    return res, list(fin)[:n], list(peak)[:n]


def hh_sim_weighted_mean(values, counts) -> float:
    n = len(values)
    v = (C.c_double * max(n, 1))(*values)
    c = (C.c_int64 * max(n, 1))(*[int(t) for t in counts])
    out = C.c_double()
    _check(lib.hh_sim_weighted_mean(v, c, n, C.byref(out)))
    return out.value


def hh_plan_layers(stages: Sequence[hh_sim_stage], total_layers, n_micro, micro_batch, seq, hidden, data_parallel,
                   flop_per_layer, slack=2):
    """-> (layers per stage, hh_sim_result of that split)"""
    n = len(stages)
    arr = (hh_sim_stage * max(n, 1))(*stages)
    out = (C.c_int32 * max(n, 1))()
    res = hh_sim_result()
    _check(lib.hh_plan_layers(arr, n, total_layers, n_micro, micro_batch, seq, hidden, data_parallel, float(flop_per_layer), slack,
                              out, C.byref(res)))
    return list(out)[:n], res


def hh_plan_order(groups: Sequence[hh_sim_stage], counts: Sequence[int], cross_link_gbytes_per_s, total_layers, n_micro,
                  micro_batch, seq, hidden, data_parallel, flop_per_layer, slack=2):
    """-> (group index per pipeline position, layers per stage in pipeline order, hh_sim_result)"""
    n = len(groups)
    assert len(counts) == n
    arr = (hh_sim_stage * max(n, 1))(*groups)
    cnt = (C.c_int32 * max(n, 1))(*counts)
    total = max(sum(c for c in counts if c > 0), 1)
    order = (C.c_int32 * max(n, 1))()
    layers = (C.c_int32 * total)()
    res = hh_sim_result()
    _check(lib.hh_plan_order(arr, cnt, n, float(cross_link_gbytes_per_s), total_layers, n_micro, micro_batch, seq, hidden,
                             data_parallel, float(flop_per_layer), slack, order, layers, C.byref(res)))
    return list(order)[:n], list(layers)[:sum(counts)], res


def hh_plan_cluster(groups: Sequence[hh_cluster_group], cross_link_gbytes_per_s, total_layers, global_batch, micro_batch, seq,
                    hidden, flop_per_layer, slack=2, max_stages=4096):
    """-> (hh_cluster_plan, layers per stage in pipeline order)"""
    n = len(groups)
    arr = (hh_cluster_group * max(n, 1))(*groups)
    plan = hh_cluster_plan()
    layers = (C.c_int32 * max_stages)()
    _check(lib.hh_plan_cluster(arr, n, float(cross_link_gbytes_per_s), total_layers, global_batch, micro_batch, seq, hidden,
                               float(flop_per_layer), slack, C.byref(plan), layers, max_stages))
    return plan, list(layers)[:plan.n_stages]
