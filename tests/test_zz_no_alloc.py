"""The forward entry point that allocates nothing (hh_layer_fwd_noalloc) against hh_layer_fwd, through the C-ABI:
two calls in a row on the library's one scratch array, the second with a smaller input, each bit for bit; plus its
two refusals (no rotary table yet, shape too large for the array)."""
import sys

import numpy as np
import pytest
import torch

from paper_2405_16256_amd import binding as hh
from paper_2405_16256_amd import inputs as I
from paper_2405_16256_amd import glue as L

pytestmark = pytest.mark.gpu


def reference_forward(ctx, cfg, layer, x):
    saved_b, ws_b = hh.hh_layer_sizes(cfg)
    y = torch.empty_like(x)
    ws = torch.empty(saved_b + ws_b, dtype=torch.uint8, device=L.DEV)
    hh.hh_layer_fwd(ctx, cfg, layer.wstruct, x, y, None, ws, L.stream_ptr())
    torch.cuda.synchronize()
    return y


def test_forward_without_allocation_matches_the_ordinary_forward_twice_in_a_row():
    ctx = hh.hh_ctx_create(0)
    try:
        shapes = [(I.LayerShape(1024, 8, 128, 2048, 700, 1, n_kv_heads=2), True, 501),
                  (I.LayerShape(256, 2, 128, 320, 200, 1), True, 502),                     # smaller, right after
                  (I.LayerShape(72, 2, 64, 88, 37, 2), False, 503)]                        # fp32 path
        # one reservation that covers every call below: the longest sequence, same head size and base
        for s, bf16, seed in shapes:
            cfg = L.cfg_of(s, bf16)
            need = sum(hh.hh_layer_sizes(cfg))
            assert need <= hh.HH_STATIC_SCRATCH_BYTES, (s, need)
            print("[case] no-alloc forward shape=%s bf16=%s scratch needed %.1f MB" % (s, bf16, need / 1e6), file=sys.stderr, flush=True)
            w = I.layer_weights(seed, 0, s, bf16)
            x_np, _ = I.activations(seed, s, 0, bf16)
            layer = L.DeviceLayer(w, s, bf16)
            x = L.to_dev(x_np, bf16)
            hh.hh_ctx_reserve(ctx, cfg)
            want = reference_forward(ctx, cfg, layer, x)
            y = torch.full_like(x, float("nan"))
            hh.hh_layer_fwd_noalloc(ctx, cfg, layer.wstruct, x, y, L.stream_ptr())
            torch.cuda.synchronize()
            assert torch.equal(y, want), s
            # and once more on the same array, which now holds this call's leftovers
            y.fill_(float("nan"))
            hh.hh_layer_fwd_noalloc(ctx, cfg, layer.wstruct, x, y, L.stream_ptr())
            torch.cuda.synchronize()
            assert torch.equal(y, want), s
    finally:
        torch.cuda.synchronize()
        hh.hh_ctx_destroy(ctx)


def test_forward_without_allocation_refuses_what_it_cannot_do():
    ctx = hh.hh_ctx_create(0)
    try:
        s = I.LayerShape(256, 2, 128, 320, 64, 1)
        cfg = L.cfg_of(s, True)
        layer = L.DeviceLayer(I.layer_weights(504, 0, s, True), s, True)
        x = L.to_dev(I.activations(504, s, 0, True)[0], True)
        y = torch.empty_like(x)
        with pytest.raises(hh.HHError) as e:          # a fresh context has no rotary table and this call may not build one
            hh.hh_layer_fwd_noalloc(ctx, cfg, layer.wstruct, x, y, L.stream_ptr())
        assert e.value.code == hh.HH_ERR_INVALID_ARG and "hh_ctx_reserve" in str(e.value)
        hh.hh_ctx_reserve(ctx, cfg)
        hh.hh_layer_fwd_noalloc(ctx, cfg, layer.wstruct, x, y, L.stream_ptr())
        torch.cuda.synchronize()
        # the 140B-class share needs about 1 GB of scratch: refused before anything is enqueued (pointers are never touched)
        big = L.cfg_of(I.CFG3, True)
        hh.hh_ctx_reserve(ctx, big)
        assert sum(hh.hh_layer_sizes(big)) > hh.HH_STATIC_SCRATCH_BYTES
        with pytest.raises(hh.HHError) as e:
            hh.hh_layer_fwd_noalloc(ctx, big, layer.wstruct, x, y, L.stream_ptr())
        assert e.value.code == hh.HH_ERR_BUFFER_TOO_SMALL
    finally:
        torch.cuda.synchronize()
        hh.hh_ctx_destroy(ctx)
