#!/usr/bin/env python3
"""Decoder-layer forward+backward throughput on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
hh_stage_step over the workload's layers and micro-batches (for the default
workload, one 140B-class TP=8-share decoder layer, one micro-batch of 4096
tokens: forward, then backward with fp32 gradient accumulation), every kernel
hand-written HIP behind the C-ABI.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3|cfg2|cfg4|cfg4-1f1b|13b|h8192-tp8|h8192-gqa-tp8|h8192-gqa] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # dense bf16 MFMA, MI355X
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "cfg3_layer_hbm_traffic_counters.txt")
KERNEL_SOURCES = ("gemm_bf16.hip", "common.h")      # what the roofline kernel is built from


def kernel_sources_sha256():
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2405_16256_amd", "csrc", f), "rb").read())
    return h.hexdigest()


def measured_traffic(workload, family):
    """HBM-side bytes per GEMM call of the roofline family, from the rocprofv3 FETCH_SIZE / WRITE_SIZE summary kept
    under profiles/ (its last lines state workload, family, bytes and the hash of the kernel sources the counters were
    taken on).  None when there is no figure for this workload and family or the kernel has changed since."""
    try:
        for line in open(TRAFFIC_PROFILE):
            if line.startswith("bench_roofline_traffic "):
                kv = dict(t.split("=", 1) for t in line.split()[1:])
                if kv.get("workload") == workload and kv.get("family") == family and kv.get("kernel_sources_sha256") == kernel_sources_sha256():
                    return float(kv["bytes_per_launch"])
    except OSError:
        pass
    return None


def workloads():
    from paper_2405_16256_amd import inputs as I
    return {
        "cfg2": dict(shape=I.CFG2, k=1, M=1, seed=I.SEEDS["cfg2"],
                     name="cfg2: 7B-class decoder layer, hidden 4096, 32x128 heads, ffn 11008, seq 2048, micro-batch 1, bf16 fwd+bwd"),
        "cfg3": dict(shape=I.CFG3, k=1, M=1, seed=I.SEEDS["cfg3"],
                     name="cfg3: 140B-class decoder layer at a TP=8 share, hidden 12288, 12x128 local heads, local ffn 4096, "
                          "seq 4096, micro-batch 1, bf16 fwd+bwd"),
        "13b": dict(shape=I.SHAPE_13B, k=1, M=1, seed=61,
                    name="13B-class decoder layer, hidden 5120, 40x128 heads, ffn 13824, seq 2048, micro-batch 1, bf16 fwd+bwd"),
        "h8192-tp8": dict(shape=I.SHAPE_70B_TP8, k=1, M=1, seed=62,
                          name="hidden-8192 (70B/140B-class of Table 1) decoder layer at a TP=8 share, 8x128 local heads, local ffn 3584, "
                               "seq 4096, micro-batch 1, bf16 fwd+bwd"),
        "h8192-gqa-tp8": dict(shape=I.SHAPE_70B_GQA_TP8, k=1, M=1, seed=63,
                              name="hidden-8192 decoder layer with grouped-query attention at a TP=8 share, 8 local query heads on 1 local "
                                   "key/value head (d 128), local ffn 3584, seq 4096, micro-batch 1, bf16 fwd+bwd"),
        "h8192-gqa": dict(shape=I.SHAPE_70B_GQA, k=1, M=1, seed=64,
                          name="whole hidden-8192 decoder layer (no tensor parallelism), 64 query / 8 key-value heads of 128, ffn 28672, "
                               "seq 4096, micro-batch 1, bf16 fwd+bwd"),
        "cfg4": dict(shape=I.CFG3, k=4, M=8, seed=I.SEEDS["cfg4"],
                     name="cfg4: pipeline-stage step, 4 layers of the cfg3 shape x 8 micro-batches of seq 4096, fp32 grad accumulation"),
        "cfg4-1f1b": dict(shape=I.CFG3, k=4, M=8, live=2, seed=I.SEEDS["cfg4"],
                          name="cfg4 in one-forward-one-backward order with 2 live micro-batches (activation pool a quarter of cfg4's)"),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3", choices=["cfg2", "cfg3", "cfg4", "cfg4-1f1b", "13b", "h8192-tp8", "h8192-gqa-tp8", "h8192-gqa"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-trace", action="store_true", help="do not time kernel families with events (no roofline object)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the two side figures of the default workload: the 4-layer x 8-micro-batch stage step against 32 "
                         "single-layer passes, and the oracle timed on the tiny and the 7B-class configuration")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device copy (a kernel of known HBM traffic) for scaling rocprofv3 byte counters")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: the library runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported" % a.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2405_16256_amd import binding as hh
    from paper_2405_16256_amd import inputs as I
    from paper_2405_16256_amd import glue as L

    wl = workloads()[a.workload]
    s, k, M, seed = wl["shape"], wl["k"], wl["M"], wl["seed"]
    torch.cuda.set_device(0)
    cfg = L.cfg_of(s, True)
    ctx = hh.hh_ctx_create(0)
    hh.hh_ctx_reserve(ctx, cfg)

    t0 = time.time()
    w_np = [I.layer_weights(seed, l, s, True) for l in range(k)]
    layers = [L.DeviceLayer(w, s, True) for w in w_np]
    acts = [I.activations(seed, s, m, True) for m in range(min(M, 2))]   # micro-batches beyond 2 reuse these draws
    xs = [L.to_dev(acts[m % len(acts)][0], True) for m in range(M)]
    dys = [L.to_dev(acts[m % len(acts)][1], True) for m in range(M)]
    ys = [torch.empty_like(t) for t in xs]
    dxs = [torch.empty_like(t) for t in xs]
    live = wl.get("live", M)
    pool_b, ws_b = hh.hh_stage_sizes(cfg, k, live)
    pool = torch.empty(pool_b, dtype=torch.uint8, device=L.DEV)
    wsp = torch.empty(ws_b, dtype=torch.uint8, device=L.DEV)
    print("[bench] inputs ready in %.1fs; pool %.2f GB" % (time.time() - t0, pool_b / 1e9), file=sys.stderr, flush=True)

    wst, gst = [l.wstruct for l in layers], [l.gstruct for l in layers]
    st = L.stream_ptr()

    def step(stream=st):
        # steady-state training: gradients accumulate, nothing is zeroed inside the timed region
        if live == M:
            hh.hh_stage_step(ctx, cfg, wst, xs, ys, dys, dxs, gst, 0, pool, wsp, stream)
        else:
            hh.hh_stage_step_1f1b(ctx, cfg, wst, live, xs, ys, dys, dxs, gst, 0, pool, wsp, stream)

    if a.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=L.DEV).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)            # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst
    # Warm-up steps run with every kernel family bracketed by events: this gives the per-family breakdown and
    # names the dominant GEMM family.  In the timed region only that family is bracketed, because each event
    # between two kernels costs a few microseconds (28 launches per layer pass).
    fam_all = {}
    traced_warm = a.warmup - 1 if not a.no_trace else 0     # the very first step pays one-time costs: not traced
    for i in range(a.warmup):
        if i == 1 and traced_warm > 0:
            torch.cuda.synchronize()
            hh.hh_trace_begin(ctx, traced_warm * k * M * 40)
        step()
    torch.cuda.synchronize()
    if traced_warm > 0:
        fam_all = hh.hh_trace_end(ctx)
    dom = None
    if not a.no_trace:
        gemms = {n: v for n, v in fam_all.items() if n.startswith("gemm") and v[0] > 0}
        dom = max(gemms, key=lambda n: gemms[n][1]) if gemms else "gemm_tn"
        hh.hh_trace_begin(ctx, a.steps * k * M * 8, [dom])
    # one event per step boundary on the stream the library launches on (torch's current stream): per-step
    # durations for the median; the mean comes from the host clock around the whole region
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(a.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(a.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    fam = hh.hh_trace_end(ctx) if not a.no_trace else {}
    per_step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(a.steps))
    median_ms = per_step_ms[len(per_step_ms) // 2] if len(per_step_ms) % 2 else 0.5 * (per_step_ms[len(per_step_ms) // 2 - 1] + per_step_ms[len(per_step_ms) // 2])

    f, b = hh.hh_layer_flops(cfg)
    flop_step = (f + b) * k * M
    ms = dt / a.steps * 1e3
    tflops = flop_step / (dt / a.steps) / 1e12
    tokens_s = s.tokens * M / (dt / a.steps)

    roofline = None
    breakdown = {n: {"launches": v[0], "ms_per_step": round(v[1] / traced_warm, 4),
                     ("GB_per_s" if n == "elementwise" else "tflops"): round(v[2] / (v[1] * 1e-3) / (1e9 if n == "elementwise" else 1e12), 1)}
                 for n, v in fam_all.items() if v[0] > 0}
    if dom is not None and fam[dom][0] > 0:
        launches, dms, dwork = fam[dom]
        achieved = dwork / (dms * 1e-3) / 1e12
        traffic = measured_traffic(a.workload, dom)
        roofline = {"kernel": "k_gemm_dma (%s; one launch = one GEMM call incl. its k-split tail)" % dom, "bound": "mfma",
                    "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                    "traffic_unit": "bytes per launch",
                    "traffic_source": "profiles/" + os.path.basename(TRAFFIC_PROFILE) + ("" if traffic is not None else " holds no counter pass of this kernel build"),
                    "launches": launches,
                    "avg_launch_ms": round(dms / launches, 4), "flop_per_launch": dwork / launches,
                    "ms_per_step": round(dms / a.steps, 4)}

    out = {
        "metric": "decoder-layer fwd+bwd TFLOP/s on 1 GPU", "value": round(tflops, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms, 4), "ms_per_step_median": round(median_ms, 4),
        "ms_per_step_min_max": [round(per_step_ms[0], 4), round(per_step_ms[-1], 4)],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl["name"], "layers": k, "micro_batches": M, "live_micro_batches": live, "activation_pool_bytes": pool_b, "tokens_per_micro_batch": s.tokens,
                   "model_flop_per_step": flop_step},
        "tokens_per_s": round(tokens_s, 1),
        "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "roofline": roofline,
        "kernel_families_warmup_steps": breakdown,
    }

    if not a.no_cpu_baseline:
        # the oracle, as it stands, on the host cores: one full layer forward+backward of the same workload
        from oracle import decoder_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        x0, dy0 = acts[0]
        t0 = time.perf_counter()
        yo, cache = O.layer_forward(x0, w_np[0], s.n_heads, s.head_dim, s.rms_eps, s.rope_base, s.kv_heads)
        dxo, go = O.layer_backward(dy0, w_np[0], cache)
        ct = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round((f + b) / ct / 1e12, 4), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                               "sample": "one layer x one micro-batch of the same workload (fp64, %.1f s)" % ct}
        # the run also serves as an end-to-end parity check of the timed configuration
        err = L.rel_err(L.to_np(ys[0]), yo) if k == 1 else None
        out["parity_y_rel_fro"] = None if err is None else float("%.3e" % err)
    if a.workload == "cfg3" and not a.no_extras:
        out["graph_replay"] = graph_replay(L, step, a.steps, flop_step)
        out["stage_step_cfg4"] = stage_step_ratio(hh, I, L, ctx, median_ms)
        if not a.no_cpu_baseline:
            out["cpu_baseline_other_configs"] = oracle_times(I)
    print(json.dumps(out), flush=True)
    hh.hh_ctx_destroy(ctx)


def graph_replay(L, step, steps, flop_step):
    """The same step recorded once into a HIP graph on a side stream and replayed `steps` times: what a caller who
    captures the library's launches saves on launch gaps.  Reported beside the eager figure, never as `value`."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(L.stream_ptr())
        torch.cuda.synchronize()
        graph.replay()                               # first replay untimed
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    return {"ms_per_step": round(ms, 4), "steps": steps, "tflops": round(flop_step / (ms * 1e-3) / 1e12, 1)}


def stage_step_ratio(hh, I, L, ctx, layer_ms):
    """The pipeline-stage workload (4 layers x 8 micro-batches of the default layer shape) in one hh_stage_step call,
    against 32 times the single-layer step measured just before: what the stage scheduler adds."""
    import torch
    wl = workloads()["cfg4"]
    s, k, M, seed = wl["shape"], wl["k"], wl["M"], wl["seed"]
    cfg = L.cfg_of(s, True)
    layers = [L.DeviceLayer(I.layer_weights(seed, l, s, True), s, True) for l in range(k)]
    acts = [I.activations(seed, s, m, True) for m in range(2)]
    xs = [L.to_dev(acts[m % 2][0], True) for m in range(M)]
    dys = [L.to_dev(acts[m % 2][1], True) for m in range(M)]
    ys = [torch.empty_like(t) for t in xs]
    dxs = [torch.empty_like(t) for t in xs]
    pool_b, ws_b = hh.hh_stage_sizes(cfg, k, M)
    pool = torch.empty(pool_b, dtype=torch.uint8, device=L.DEV)
    wsp = torch.empty(ws_b, dtype=torch.uint8, device=L.DEV)
    wst, gst = [l.wstruct for l in layers], [l.gstruct for l in layers]
    st = L.stream_ptr()
    times = []
    for i in range(5):                          # first one untimed
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record()
        hh.hh_stage_step(ctx, cfg, wst, xs, ys, dys, dxs, gst, 0, pool, wsp, st)
        a1.record()
        torch.cuda.synchronize()
        if i:
            times.append(a0.elapsed_time(a1))
    times.sort()
    ms = 0.5 * (times[1] + times[2])
    f, b = hh.hh_layer_flops(cfg)
    return {"workload": wl["name"], "ms_per_step_median_of_4": round(ms, 3), "tflops": round((f + b) * k * M / (ms * 1e-3) / 1e12, 1),
            "tokens_per_s": round(s.tokens * M / (ms * 1e-3), 1), "single_layer_ms_median": round(layer_ms, 4),
            "step_over_32_layer_passes": round(ms / (k * M * layer_ms), 4)}


def oracle_times(I):
    """The oracle, as it stands, on one layer forward+backward of the tiny fp32 configuration (median of 5) and of the
    7B-class configuration (one run): the reported CPU baseline of the other layer configurations."""
    from oracle import decoder_oracle as O
    res = {}
    for name, s, bf16, reps in (("cfg1", I.CFG1, False, 5), ("cfg2", I.CFG2, True, 1)):
        w = I.layer_weights(I.SEEDS[name], 0, s, bf16)
        x, dy = I.activations(I.SEEDS[name], s, 0, bf16)
        ts = []
        for _ in range(reps):
            t0 = time.perf_counter()
            _, cache = O.layer_forward(x, w, s.n_heads, s.head_dim, s.rms_eps, s.rope_base, s.kv_heads)
            O.layer_backward(dy, w, cache)
            ts.append(time.perf_counter() - t0)
        ts.sort()
        t = ts[len(ts) // 2]
        flop = 3.0 * (s.tokens * (2.0 * (s.attn + 2 * s.attn_kv + s.attn) * s.hidden + 6.0 * s.hidden * s.ffn) +
                      4.0 * s.head_dim * s.micro_batch * s.n_heads * (s.seq * (s.seq + 1) / 2))
        res[name] = {"seconds": round(t, 4), "tflops_fp64": round(flop / t / 1e12, 4), "runs": reps}
    return res


if __name__ == "__main__":
    main()
