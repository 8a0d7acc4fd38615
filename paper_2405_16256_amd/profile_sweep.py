"""Per-layer profile sweep for the performance predictor (Section 3.2 of the paper: the predictor is
fed with the measured computation time of a layer on each accelerator type).

For the 7B-class and the 140B-class TP-share layer shapes, at seq {1024, 2048, 4096} x micro-batch
{1, 2, 4} and a stage depth of 1..12 layers, runs hh_layer_profile and prints one JSON line per
(shape, seq, micro-batch, depth) with the per-layer forward / backward milliseconds and TFLOP/s and the
byte figures of the profile record.  Every layer of a stage has its own seeded weights and its own fp32
gradient buffers, as in a real stage (12 layers of the 140B-class share hold 16 GB of them).

  python -m paper_2405_16256_amd.profile_sweep [--depths 1,4,12] [--iters 3] [--quick]
"""
from __future__ import annotations

import argparse
import json
import sys

import torch

from . import binding as hh
from . import glue as L
from . import inputs as I


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--depths", default="1,2,4,8,12")
    ap.add_argument("--iters", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--quick", action="store_true", help="seq 1024/4096, micro-batch 1/4 only")
    a = ap.parse_args()
    depths = [int(d) for d in a.depths.split(",")]
    seqs = [1024, 4096] if a.quick else [1024, 2048, 4096]
    mbs = [1, 4] if a.quick else [1, 2, 4]
    ctx = hh.hh_ctx_create(0)
    seed = I.SEEDS["cfg5"]
    for name, base in (("7B-class", I.CFG2), ("140B-class TP=8 share", I.CFG3)):
        layers = [L.DeviceLayer(I.layer_weights(seed, l, base, True), base, True) for l in range(max(depths))]
        for S in seqs:
            for B in mbs:
                s = I.LayerShape(base.hidden, base.n_heads, base.head_dim, base.ffn, S, B)
                cfg = L.cfg_of(s, True)
                x_np, dy_np = I.activations(seed, s, 0, True)
                x, dy = L.to_dev(x_np, True), L.to_dev(dy_np, True)
                for k in depths:
                    pool_b, ws_b = hh.hh_stage_sizes(cfg, k, 1)
                    pool = torch.empty(pool_b, dtype=torch.uint8, device=L.DEV)
                    wsp = torch.empty(ws_b, dtype=torch.uint8, device=L.DEV)
                    recs = hh.hh_layer_profile(ctx, cfg, [l.wstruct for l in layers[:k]], [l.gstruct for l in layers[:k]], x, dy, a.warmup,
                                               a.iters, pool, wsp, L.stream_ptr())
                    f = [r.fwd_ms for r in recs]
                    b = [r.bwd_ms for r in recs]
                    r0 = recs[0]
                    print(json.dumps({
                        "shape": name, "seq": S, "micro_batch": B, "depth": k,
                        "fwd_ms_per_layer": [round(v, 4) for v in f], "bwd_ms_per_layer": [round(v, 4) for v in b],
                        "fwd_ms_mean": round(sum(f) / k, 4), "bwd_ms_mean": round(sum(b) / k, 4),
                        "fwd_tflops": round(r0.fwd_flop / (sum(f) / k * 1e-3) / 1e12, 1),
                        "bwd_tflops": round(r0.bwd_flop / (sum(b) / k * 1e-3) / 1e12, 1),
                        "weight_bytes": r0.weight_bytes, "grad_bytes": r0.grad_bytes,
                        "saved_act_bytes": r0.saved_act_bytes, "p2p_bytes": r0.p2p_bytes,
                        "workspace_bytes": r0.workspace_bytes}), flush=True)
                    del pool, wsp
                del x, dy
        del layers
        torch.cuda.empty_cache()
    hh.hh_ctx_destroy(ctx)


if __name__ == "__main__":
    sys.exit(main())
