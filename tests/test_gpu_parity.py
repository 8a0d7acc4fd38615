"""GPU parity: the HIP path, called through the C-ABI, against the CPU fp64 oracle on
the same seeded inputs, tensor by tensor, in relative Frobenius norm.

Tolerances (from the workload statement): fp32 path 1e-4 on every tensor; bf16
path 2e-2 on outputs, 5e-2 on gradients.  A healthy bf16 run sits near 3e-3..8e-3,
so anything above 1.5e-2 is printed as suspicious even though it passes.
"""
import sys
import time

import numpy as np
import pytest
import torch

from oracle import decoder_oracle as O
from paper_2405_16256_amd import binding as hh
from paper_2405_16256_amd import inputs as I
from paper_2405_16256_amd import glue as L

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16_OUT = 2e-2
TOL_BF16_GRAD = 5e-2


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def ctx():
    c = hh.hh_ctx_create(0)
    yield c
    torch.cuda.synchronize()
    hh.hh_ctx_destroy(c)


def block_errors(got, ref, br, bc):
    """Largest relative Frobenius error over the br x bc blocks of a 2-D array (ragged edge blocks included)."""
    R, C = ref.shape
    nr, nc = -(-R // br), -(-C // bc)
    d2 = np.zeros((nr * br, nc * bc))
    r2 = np.zeros((nr * br, nc * bc))
    d2[:R, :C] = (got - ref) ** 2
    r2[:R, :C] = ref ** 2
    num = d2.reshape(nr, br, nc, bc).sum(axis=(1, 3))
    den = r2.reshape(nr, br, nc, bc).sum(axis=(1, 3))
    return float(np.sqrt(np.max(num / np.where(den > 0, den, 1.0))))


def saved_tensor(saved, cfg, name, rows, cols, bf16):
    """One of the tensors hh_layer_fwd leaves in the saved block, as fp64 [rows, cols]."""
    off = getattr(hh.hh_saved_layout_of(cfg), name)
    es = 2 if bf16 else 4
    raw = saved[off:off + rows * cols * es]
    return L.to_np(raw.view(torch.bfloat16 if bf16 else torch.float32).reshape(rows, cols))


def check_layer(ctx, s, bf16, seed, packed=True, label=""):
    say("[case] %s shape=%s bf16=%s packed=%s seed=%d" % (label, s, bf16, packed, seed))
    w = I.layer_weights(seed, 0, s, bf16)
    x, dy = I.activations(seed, s, 0, bf16)
    layer = L.DeviceLayer(w, s, bf16, packed)
    t0 = time.time()
    y, dx, saved = L.run_layer(ctx, s, bf16, layer, x, dy)
    g = layer.grads_np()
    T, H = s.tokens, s.hidden
    h = saved_tensor(saved, L.cfg_of(s, bf16), "h", T, H, bf16)
    say("  gpu done %.2fs; oracle..." % (time.time() - t0))
    t0 = time.time()
    yo, cache = O.layer_forward(x, w, s.n_heads, s.head_dim, s.rms_eps, s.rope_base, s.kv_heads)
    dxo, go = O.layer_backward(dy, w, cache)
    say("  oracle done %.1fs" % (time.time() - t0))
    return judge_layer(s, bf16, x, y, dx, g, h, yo, dxo, go, cache["h"])


def judge_layer(s, bf16, x, y, dx, g, h, yo, dxo, go, ho, scale=1.0):
    """Every tensor of one layer pass against the oracle's, at the stated tolerances (times `scale`)."""
    tol_out = (TOL_BF16_OUT if bf16 else TOL_F32) * scale
    tol_grad = (TOL_BF16_GRAD if bf16 else TOL_F32) * scale
    T, H = s.tokens, s.hidden
    x2 = np.asarray(x, dtype=np.float64).reshape(T, H)
    errs = {"y": L.rel_err(y, yo), "dx": L.rel_err(dx, dxo)}
    for n in I.WEIGHT_NAMES:
        errs["d" + n] = L.rel_err(g[n], go[n])
    # the residual must not hide a broken branch: both branch outputs are judged against their own norms
    branch = {"y-x": L.rel_err(y.reshape(T, H) - x2, yo.reshape(T, H) - x2), "h-x": L.rel_err(h - x2, ho.reshape(T, H) - x2),
              "y-h": L.rel_err(y.reshape(T, H) - h, (yo - ho).reshape(T, H))}
    say("  errors: " + " ".join("%s=%.2e" % kv for kv in errs.items()) + " | branches " + " ".join("%s=%.2e" % kv for kv in branch.items()))
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(dx))
    assert errs["y"] <= tol_out, errs
    for n, e in errs.items():
        if n != "y":
            assert e <= tol_grad, (n, errs)
    # allowance for the rounding of the bf16 residual stream the branch is a difference of (3 half-ulps of the
    # stream, which is large next to a small branch)
    for n, (big, small) in {"y-x": (yo, yo.reshape(T, H) - x2), "h-x": (ho, ho.reshape(T, H) - x2)}.items():
        floor = 3.0 * 2.0 ** -9 * np.linalg.norm(big) / np.linalg.norm(small)
        assert branch[n] <= (max(0.05, floor) * scale if bf16 else 1e-3), (n, branch, floor)
    # block by block: a single wrong tile or row block must not drown in the norm of a large tensor
    blocks = {}
    if T * H >= 64 * 128 * 128:
        blocks["y/128rows"] = (block_errors(y.reshape(T, H), yo.reshape(T, H), 128, H), tol_out)
        blocks["dx/128rows"] = (block_errors(dx.reshape(T, H), dxo.reshape(T, H), 128, H), tol_grad)
    for n in I.WEIGHT_NAMES:
        if go[n].ndim == 2 and go[n].size >= 64 * 256 * 256:
            blocks["d%s/256x256" % n] = (block_errors(g[n], go[n], 256, 256), tol_grad)
    if blocks:
        say("  worst block: " + " ".join("%s=%.2e" % (n, e) for n, (e, _) in blocks.items()))
        for n, (e, tol) in blocks.items():
            assert e <= tol, (n, e, tol)
    return errs


# ------------------------------------------------------------------ fp32 path
def test_fp32_tiny_config(ctx):
    check_layer(ctx, I.CFG1, False, I.SEEDS["cfg1"], label="cfg1")


def test_fp32_ragged_unpacked(ctx):
    check_layer(ctx, I.LayerShape(72, 2, 64, 88, 37, 2), False, 11, packed=False, label="f32-ragged")


def test_fp32_head_dim_128_single_token(ctx):
    check_layer(ctx, I.LayerShape(128, 1, 128, 40, 1, 3), False, 12, label="f32-S1")


# ------------------------------------------------------------------ bf16 path
def test_bf16_small_ragged(ctx):
    check_layer(ctx, I.LayerShape(256, 2, 128, 320, 200, 2), True, 21, label="bf16-small")


def test_bf16_small_unpacked_weights(ctx):
    check_layer(ctx, I.LayerShape(256, 2, 128, 320, 200, 2), True, 21, packed=False, label="bf16-unpacked")


def test_bf16_head_dim_64(ctx):
    check_layer(ctx, I.LayerShape(192, 3, 64, 256, 130, 1), True, 22, label="bf16-d64")


def test_bf16_single_token_and_exact_tiles(ctx):
    check_layer(ctx, I.LayerShape(128, 1, 128, 64, 1, 1), True, 23, label="bf16-S1")
    check_layer(ctx, I.LayerShape(128, 2, 64, 128, 128, 2), True, 24, label="bf16-exact")


def test_bf16_mid_ragged_large_tiles(ctx):
    # enough 256x256 output tiles to take the large-tile GEMM kernels in all three forms, ragged T
    check_layer(ctx, I.LayerShape(4096, 8, 128, 4096, 3300, 1), True, 25, label="bf16-mid")


def test_bf16_7b_class_layer_full_size(ctx):
    check_layer(ctx, I.CFG2, True, I.SEEDS["cfg2"], label="cfg2")


def test_bf16_140b_class_tp_share_full_size(ctx):
    check_layer(ctx, I.CFG3, True, I.SEEDS["cfg3"], label="cfg3")


def test_bf16_head_dim_64_long_ragged_sequence(ctx):
    # S = 1100 (ragged) with few workgroups: attention forward and dQ run with the key tiles split between two
    # wave groups, here for head_dim 64
    check_layer(ctx, I.LayerShape(512, 8, 64, 1024, 1100, 1), True, 63, label="d64-long")


def test_bf16_13b_class_layer_full_size(ctx):
    # hidden 5120 (Table 1): 20 x 20 tiles of 256 leave k-split tails in every GEMM family
    check_layer(ctx, I.SHAPE_13B, True, 61, label="13b")


def test_bf16_hidden_8192_tp_share_two_samples(ctx):
    # the 70B / 140B hidden size of Table 1 at a TP=8 share, two samples of 2048 tokens
    s = I.SHAPE_70B_TP8
    check_layer(ctx, I.LayerShape(s.hidden, s.n_heads, s.head_dim, s.ffn, 2048, 2), True, 62, label="h8192-tp8")


def test_bf16_profile_sweep_spot_points_with_several_samples(ctx):
    # the two points of the per-layer profile sweep that are checked against the oracle: more than one sample per
    # micro-batch at the 7B-class and at the 140B-class TP-share shape
    s = I.CFG2
    check_layer(ctx, I.LayerShape(s.hidden, s.n_heads, s.head_dim, s.ffn, 1024, 2), True, I.SEEDS["cfg5"], label="cfg5: cfg2 shape S=1024 B=2")
    s = I.CFG3
    check_layer(ctx, I.LayerShape(s.hidden, s.n_heads, s.head_dim, s.ffn, 1024, 4), True, I.SEEDS["cfg5"] + 1, label="cfg5: cfg3 shape S=1024 B=4")


# ------------------------------------------------------------- determinism
def test_two_runs_are_bit_identical(ctx):
    s = I.LayerShape(256, 2, 128, 320, 200, 2)
    w = I.layer_weights(31, 0, s, True)
    x, dy = I.activations(31, s, 0, True)
    outs = []
    for _ in range(2):
        layer = L.DeviceLayer(w, s, True)
        y, dx, _ = L.run_layer(ctx, s, True, layer, x, dy)
        outs.append((y, dx, layer.grads_np()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])
    for n in I.WEIGHT_NAMES:
        assert np.array_equal(outs[0][2][n], outs[1][2][n]), n


def test_accumulate_adds_to_existing_gradients(ctx):
    s = I.LayerShape(128, 2, 64, 128, 96, 1)
    w = I.layer_weights(32, 0, s, True)
    x, dy = I.activations(32, s, 0, True)
    layer = L.DeviceLayer(w, s, True)
    L.run_layer(ctx, s, True, layer, x, dy, accumulate=False)
    g1 = layer.grads_np()
    L.run_layer(ctx, s, True, layer, x, dy, accumulate=True)
    g2 = layer.grads_np()
    for n in I.WEIGHT_NAMES:
        np.testing.assert_allclose(g2[n], 2 * g1[n], rtol=1e-6, atol=1e-7, err_msg=n)
    # overwrite mode ignores what the buffers held
    for n in I.WEIGHT_NAMES:
        layer.g[n].fill_(1e6)
    L.run_layer(ctx, s, True, layer, x, dy, accumulate=False)
    g3 = layer.grads_np()
    for n in I.WEIGHT_NAMES:
        assert np.array_equal(g3[n], g1[n]), n


# ------------------------------------------------------------------ stage step
def run_stage(ctx, s, bf16, seed, k, M, zero_first=True):
    cfg = L.cfg_of(s, bf16)
    ws_np = [I.layer_weights(seed, l, s, bf16) for l in range(k)]
    acts = [I.activations(seed, s, m, bf16) for m in range(M)]
    layers = [L.DeviceLayer(w, s, bf16) for w in ws_np]
    xs = [L.to_dev(a[0], bf16) for a in acts]
    dys = [L.to_dev(a[1], bf16) for a in acts]
    ys = [torch.empty_like(t) for t in xs]
    dxs = [torch.empty_like(t) for t in xs]
    pool_b, wsb = hh.hh_stage_sizes(cfg, k, M)
    pool = torch.empty(pool_b, dtype=torch.uint8, device=L.DEV)
    wsp = torch.empty(wsb, dtype=torch.uint8, device=L.DEV)
    hh.hh_stage_step(ctx, cfg, [l.wstruct for l in layers], xs, ys, dys, dxs, [l.gstruct for l in layers],
                     zero_first, pool, wsp, L.stream_ptr())
    torch.cuda.synchronize()
    return ws_np, acts, layers, ys, dxs


@pytest.mark.parametrize("bf16,shape,k,M", [
    (False, I.LayerShape(64, 1, 64, 72, 33, 1), 2, 3),
    (True, I.LayerShape(256, 4, 64, 704, 128, 1), 4, 8),     # tiny-config dims (ffn rounded to 64) in bf16, k=4, M=8
    (True, I.LayerShape(256, 2, 128, 320, 200, 2), 2, 2),
])
def test_stage_step_matches_oracle(ctx, bf16, shape, k, M):
    s = shape
    say("[case] stage bf16=%s shape=%s k=%d M=%d" % (bf16, s, k, M))
    ws_np, acts, layers, ys, dxs = run_stage(ctx, s, bf16, 41, k, M)
    yo, dxo, go = O.stage_step([a[0] for a in acts], [a[1] for a in acts], ws_np, s.n_heads, s.head_dim, s.rms_eps, s.rope_base, s.kv_heads)
    tol_out = TOL_BF16_OUT if bf16 else TOL_F32
    tol_grad = TOL_BF16_GRAD if bf16 else TOL_F32
    worst = 0.0
    for m in range(M):
        assert L.rel_err(L.to_np(ys[m]), yo[m]) <= tol_out
        assert L.rel_err(L.to_np(dxs[m]), dxo[m]) <= tol_grad
    for l in range(k):
        g = layers[l].grads_np()
        for n in I.WEIGHT_NAMES:
            e = L.rel_err(g[n], go[l][n])
            worst = max(worst, e)
            assert e <= tol_grad, (l, n, e)
    say("  worst gradient error %.2e" % worst)


def test_stage_layers_meet_the_single_layer_tolerances_on_the_tensors_the_stage_feeds_them(ctx):
    """The 140B-class TP-share shape at full size, two chained layers (hh_stage_step is these calls bit for bit).
    Each layer is judged on the inputs the stage really gives it: the oracle's layer 1 starts from the GPU's own
    layer-0 output and the oracle's layer-0 backward from the GPU's own inter-layer gradient, so every tensor of
    each layer is held to the unscaled tolerances."""
    s, bf16 = I.CFG3, True
    seed = I.SEEDS["cfg4"]
    say("[case] teacher-forced two-layer chain, shape %s" % (s,))
    cfg = L.cfg_of(s, bf16)
    ws_np = [I.layer_weights(seed, l, s, bf16) for l in range(2)]
    layers = [L.DeviceLayer(w, s, bf16) for w in ws_np]
    x_np, dy_np = I.activations(seed, s, 0, bf16)
    saved_b, ws_b = hh.hh_layer_sizes(cfg)
    x0, dy = L.to_dev(x_np, bf16), L.to_dev(dy_np, bf16)
    y0, y1, g1, g0 = (torch.empty_like(x0) for _ in range(4))
    sv = [torch.empty(saved_b, dtype=torch.uint8, device=L.DEV) for _ in range(2)]
    wsp = torch.empty(ws_b, dtype=torch.uint8, device=L.DEV)
    st = L.stream_ptr()
    hh.hh_layer_fwd(ctx, cfg, layers[0].wstruct, x0, y0, sv[0], wsp, st)
    hh.hh_layer_fwd(ctx, cfg, layers[1].wstruct, y0, y1, sv[1], wsp, st)
    hh.hh_layer_bwd(ctx, cfg, layers[1].wstruct, y0, sv[1], dy, g1, layers[1].gstruct, 0, wsp, st)
    hh.hh_layer_bwd(ctx, cfg, layers[0].wstruct, x0, sv[0], g1, g0, layers[0].gstruct, 0, wsp, st)
    torch.cuda.synchronize()
    T, H = s.tokens, s.hidden
    y0_np, y1_np, g1_np, g0_np = (L.to_np(t) for t in (y0, y1, g1, g0))
    hs = [saved_tensor(sv[l], cfg, "h", T, H, bf16) for l in range(2)]
    # layer 1 on the GPU's layer-0 output, upstream gradient dy
    yo1, c1 = O.layer_forward(y0_np, ws_np[1], s.n_heads, s.head_dim, s.rms_eps, s.rope_base, s.kv_heads)
    dxo1, go1 = O.layer_backward(dy_np, ws_np[1], c1)
    say("  layer 1 (input: the GPU's layer-0 output)")
    judge_layer(s, bf16, y0_np, y1_np, g1_np, layers[1].grads_np(), hs[1], yo1, dxo1, go1, c1["h"])
    del c1
    # layer 0 on x, upstream gradient = the GPU's layer-1 input gradient
    yo0, c0 = O.layer_forward(x_np, ws_np[0], s.n_heads, s.head_dim, s.rms_eps, s.rope_base, s.kv_heads)
    dxo0, go0 = O.layer_backward(g1_np, ws_np[0], c0)
    say("  layer 0 (upstream gradient: the GPU's layer-1 input gradient)")
    judge_layer(s, bf16, x_np, y0_np, g0_np, layers[0].grads_np(), hs[0], yo0, dxo0, go0, c0["h"])


def test_stage_step_full_shape_two_layers_two_micro_batches_vs_oracle(ctx):
    """The 140B-class TP-share shape at full size: k = 2 layers, M = 2 micro-batches of 4096 tokens, end to end
    against the oracle's own two-layer chain.

    Here the oracle's layer 1 starts from the exact layer-0 output while the GPU's starts from the bf16 one (1.2e-2 off
    at this shape, where attention scores have a standard deviation near 5), and likewise for the gradient handed
    from layer 1 to layer 0: the differences of the two layers add up, so this end-to-end comparison (and only this
    one) allows k times the single-layer tolerances.  That each layer by itself stays inside the unscaled tolerances
    on exactly these inputs is the test above; that the stage adds nothing of its own is the bit-for-bit comparison
    with chained single-layer calls below."""
    s, k, M = I.CFG3, 2, 2
    say("[case] stage full shape %s k=%d M=%d" % (s, k, M))
    ws_np, acts, layers, ys, dxs = run_stage(ctx, s, True, I.SEEDS["cfg4"], k, M)
    say("  gpu done; oracle (2 layers x 2 micro-batches)...")
    t0 = time.time()
    yo, dxo, go = O.stage_step([a[0] for a in acts], [a[1] for a in acts], ws_np, s.n_heads, s.head_dim, s.rms_eps, s.rope_base, s.kv_heads)
    say("  oracle done %.1fs" % (time.time() - t0))
    worst = {}
    for m in range(M):
        worst["y"] = max(worst.get("y", 0), L.rel_err(L.to_np(ys[m]), yo[m]))
        worst["dx"] = max(worst.get("dx", 0), L.rel_err(L.to_np(dxs[m]), dxo[m]))
    for l in range(k):
        g = layers[l].grads_np()
        per = {n: L.rel_err(g[n], go[l][n]) for n in I.WEIGHT_NAMES}
        say("  layer %d gradients: " % l + " ".join("d%s=%.2e" % kv for kv in per.items()))
        for n, e in per.items():
            worst["d" + n] = max(worst.get("d" + n, 0), e)
    say("  worst errors: " + " ".join("%s=%.2e" % kv for kv in worst.items()))
    assert worst["y"] <= k * TOL_BF16_OUT, worst
    assert all(v <= k * TOL_BF16_GRAD for v in worst.values()), worst


def test_stage_step_full_size_four_layers_eight_micro_batches_equals_chained_calls(ctx):
    """The full pipeline-stage workload (4 layers x 8 micro-batches of the 140B-class shape) through
    hh_stage_step must equal the same work done by chaining hh_layer_fwd / hh_layer_bwd, bit for bit."""
    s, k, M, bf16 = I.CFG3, 4, 8, True
    seed = I.SEEDS["cfg4"]
    say("[case] stage full size k=4 M=8 vs chained layer calls")
    cfg = L.cfg_of(s, bf16)
    ws_np = [I.layer_weights(seed, l, s, bf16) for l in range(k)]
    layers = [L.DeviceLayer(w, s, bf16) for w in ws_np]
    ref_layers = [L.DeviceLayer(w, s, bf16) for w in ws_np]
    del ws_np
    base = [I.activations(seed, s, m, bf16) for m in range(2)]          # two draws, reused with a sign flip pattern
    xs = [L.to_dev(base[m % 2][0], bf16) * (1.0 if m < 4 else -1.0) for m in range(M)]
    dys = [L.to_dev(base[m % 2][1], bf16) * (1.0 if m % 4 < 2 else 0.5) for m in range(M)]
    ys = [torch.empty_like(t) for t in xs]
    dxs = [torch.empty_like(t) for t in xs]
    pool_b, wsb = hh.hh_stage_sizes(cfg, k, M)
    say("  pool %.2f GB" % (pool_b / 1e9))
    pool = torch.empty(pool_b, dtype=torch.uint8, device=L.DEV)
    wsp = torch.empty(wsb, dtype=torch.uint8, device=L.DEV)
    st = L.stream_ptr()
    hh.hh_stage_step(ctx, cfg, [l.wstruct for l in layers], xs, ys, dys, dxs, [l.gstruct for l in layers], 1, pool, wsp, st)
    torch.cuda.synchronize()
    del pool
    saved_b, ws_b = hh.hh_layer_sizes(cfg)
    wsp2 = torch.empty(ws_b, dtype=torch.uint8, device=L.DEV)
    for m in range(M):
        t = xs[m]
        ins, saves = [], []
        for l in range(k):
            out = torch.empty_like(t)
            sv = torch.empty(saved_b, dtype=torch.uint8, device=L.DEV)
            hh.hh_layer_fwd(ctx, cfg, ref_layers[l].wstruct, t, out, sv, wsp2, st)
            ins.append(t)
            saves.append(sv)
            t = out
        assert torch.equal(t, ys[m]), m
        gdt = dys[m].clone()
        for l in reversed(range(k)):
            hh.hh_layer_bwd(ctx, cfg, ref_layers[l].wstruct, ins[l], saves[l], gdt, gdt, ref_layers[l].gstruct, m > 0, wsp2, st)
        torch.cuda.synchronize()
        assert torch.equal(gdt, dxs[m]), m
        del ins, saves
    for l in range(k):
        for n in I.WEIGHT_NAMES:
            assert torch.equal(layers[l].g[n], ref_layers[l].g[n]), (l, n)
            assert torch.isfinite(layers[l].g[n]).all()
    # the same step in one-forward-one-backward order with two live micro-batches (a quarter of the pool)
    del wsp2
    n_live = 2
    pool_b2, _ = hh.hh_stage_sizes(cfg, k, n_live)
    assert pool_b2 * M == pool_b * n_live
    say("  1F1B pool %.2f GB" % (pool_b2 / 1e9))
    pool2 = torch.empty(pool_b2, dtype=torch.uint8, device=L.DEV)
    ys2 = [torch.full_like(t, float("nan")) for t in xs]
    dxs2 = [torch.full_like(t, float("nan")) for t in xs]
    hh.hh_stage_step_1f1b(ctx, cfg, [l.wstruct for l in ref_layers], n_live, xs, ys2, dys, dxs2, [l.gstruct for l in ref_layers],
                          1, pool2, wsp, st)
    torch.cuda.synchronize()
    for m in range(M):
        assert torch.equal(ys2[m], ys[m]) and torch.equal(dxs2[m], dxs[m]), m
    for l in range(k):
        for n in I.WEIGHT_NAMES:
            assert torch.equal(layers[l].g[n], ref_layers[l].g[n]), (l, n)


@pytest.mark.parametrize("n_live", [1, 2, 3, 5])
def test_one_forward_one_backward_order_is_bit_identical_and_matches_oracle(ctx, n_live):
    """Section 2.3: 1F1B keeps at most n_live micro-batches' activations.  Backward order over micro-batches is
    the same as in the all-forward-all-backward step, so every output must be identical bit for bit."""
    s, k, M, bf16 = I.LayerShape(256, 2, 128, 320, 136, 2), 3, 5, True
    say("[case] 1F1B n_live=%d shape=%s k=%d M=%d" % (n_live, s, k, M))
    ws_np, acts, layers, ys, dxs = run_stage(ctx, s, bf16, 44, k, M)
    cfg = L.cfg_of(s, bf16)
    layers2 = [L.DeviceLayer(w, s, bf16) for w in ws_np]
    for l in layers2:                        # zero_grads_first must overwrite whatever the buffers hold
        for n in I.WEIGHT_NAMES:
            l.g[n].fill_(7.0)
    xs = [L.to_dev(a[0], bf16) for a in acts]
    dys = [L.to_dev(a[1], bf16) for a in acts]
    ys2 = [torch.full_like(t, float("nan")) for t in xs]
    dxs2 = [torch.full_like(t, float("nan")) for t in xs]
    pool_b, wsb = hh.hh_stage_sizes(cfg, k, n_live)
    full_b, _ = hh.hh_stage_sizes(cfg, k, M)
    assert pool_b * M == full_b * n_live
    pool = torch.empty(pool_b, dtype=torch.uint8, device=L.DEV)
    wsp = torch.empty(wsb, dtype=torch.uint8, device=L.DEV)
    hh.hh_stage_step_1f1b(ctx, cfg, [l.wstruct for l in layers2], n_live, xs, ys2, dys, dxs2, [l.gstruct for l in layers2], 1,
                          pool, wsp, L.stream_ptr())
    torch.cuda.synchronize()
    for m in range(M):
        assert torch.equal(ys2[m], ys[m]) and torch.equal(dxs2[m], dxs[m]), m
    for l in range(k):
        for n in I.WEIGHT_NAMES:
            assert torch.equal(layers2[l].g[n], layers[l].g[n]), (l, n)
    if n_live == 2:
        yo, dxo, go = O.stage_step([a[0] for a in acts], [a[1] for a in acts], ws_np, s.n_heads, s.head_dim, s.rms_eps,
                                   s.rope_base)
        for m in range(M):
            assert L.rel_err(L.to_np(ys2[m]), yo[m]) <= TOL_BF16_OUT
            assert L.rel_err(L.to_np(dxs2[m]), dxo[m]) <= TOL_BF16_GRAD
        for l in range(k):
            gl = layers2[l].grads_np()
            for n in I.WEIGHT_NAMES:
                e = L.rel_err(gl[n], go[l][n])
                assert e <= TOL_BF16_GRAD, (l, n, e)


def test_stage_step_equals_chained_layer_calls_bitwise(ctx):
    s, k, M, bf16 = I.LayerShape(256, 2, 128, 320, 200, 1), 3, 2, True
    ws_np, acts, layers, ys, dxs = run_stage(ctx, s, bf16, 42, k, M)
    cfg = L.cfg_of(s, bf16)
    saved_b, ws_b = hh.hh_layer_sizes(cfg)
    ref_layers = [L.DeviceLayer(w, s, bf16) for w in ws_np]
    wsp = torch.empty(ws_b, dtype=torch.uint8, device=L.DEV)
    st = L.stream_ptr()
    for m in range(M):
        t = L.to_dev(acts[m][0], bf16)
        ins, saves = [], []
        for l in range(k):
            out = torch.empty_like(t)
            sv = torch.empty(saved_b, dtype=torch.uint8, device=L.DEV)
            hh.hh_layer_fwd(ctx, cfg, ref_layers[l].wstruct, t, out, sv, wsp, st)
            ins.append(t)
            saves.append(sv)
            t = out
        assert torch.equal(t, ys[m])
        gdt = L.to_dev(acts[m][1], bf16)
        for l in reversed(range(k)):
            hh.hh_layer_bwd(ctx, cfg, ref_layers[l].wstruct, ins[l], saves[l], gdt, gdt, ref_layers[l].gstruct,
                            m > 0, wsp, st)
        torch.cuda.synchronize()
        assert torch.equal(gdt, dxs[m])
    for l in range(k):
        for n in I.WEIGHT_NAMES:
            assert torch.equal(layers[l].g[n], ref_layers[l].g[n]), (l, n)


def test_stage_step_without_zeroing_adds_to_gradients(ctx):
    s, k, M = I.LayerShape(128, 2, 64, 128, 64, 1), 2, 2
    _, _, layers_a, _, _ = run_stage(ctx, s, True, 43, k, M, zero_first=True)
    cfg = L.cfg_of(s, True)
    ws_np = [I.layer_weights(43, l, s, True) for l in range(k)]
    layers_b = [L.DeviceLayer(w, s, True) for w in ws_np]
    for lay in layers_b:
        for n in I.WEIGHT_NAMES:
            lay.g[n].fill_(3.0)
    acts = [I.activations(43, s, m, True) for m in range(M)]
    xs = [L.to_dev(a[0], True) for a in acts]
    dys = [L.to_dev(a[1], True) for a in acts]
    ys = [torch.empty_like(t) for t in xs]
    dxs = [torch.empty_like(t) for t in xs]
    pool_b, wsb = hh.hh_stage_sizes(cfg, k, M)
    pool = torch.empty(pool_b, dtype=torch.uint8, device=L.DEV)
    wsp = torch.empty(wsb, dtype=torch.uint8, device=L.DEV)
    hh.hh_stage_step(ctx, cfg, [l.wstruct for l in layers_b], xs, ys, dys, dxs, [l.gstruct for l in layers_b], 0, pool,
                     wsp, L.stream_ptr())
    torch.cuda.synchronize()
    for l in range(k):
        for n in I.WEIGHT_NAMES:
            np.testing.assert_allclose(L.to_np(layers_b[l].g[n]), L.to_np(layers_a[l].g[n]) + 3.0, rtol=2e-6, atol=1e-5)


# --------------------------------------------------------------------- profile
def test_layer_profile_records(ctx):
    s, k = I.LayerShape(512, 4, 128, 1024, 512, 2), 3
    cfg = L.cfg_of(s, True)
    layers = [L.DeviceLayer(I.layer_weights(51, l, s, True), s, True) for l in range(k)]
    x_np, dy_np = I.activations(51, s, 0, True)
    x, dy = L.to_dev(x_np, True), L.to_dev(dy_np, True)
    pool_b, wsb = hh.hh_stage_sizes(cfg, k, 1)
    pool = torch.empty(pool_b, dtype=torch.uint8, device=L.DEV)
    wsp = torch.empty(wsb, dtype=torch.uint8, device=L.DEV)
    recs = hh.hh_layer_profile(ctx, cfg, [l.wstruct for l in layers], [l.gstruct for l in layers], x, dy, 1, 3, pool, wsp,
                               L.stream_ptr())
    f, b = hh.hh_layer_flops(cfg)
    nparam = 2 * s.hidden + 4 * s.attn * s.hidden + 3 * s.ffn * s.hidden
    for l, r in enumerate(recs):
        assert r.layer == l and r.fwd_ms > 0 and r.bwd_ms > 0
        assert r.fwd_flop == f and r.bwd_flop == b
        assert abs(r.fwd_tflops - f / (r.fwd_ms * 1e-3) / 1e12) < 1e-3 * r.fwd_tflops + 1e-6
        assert r.weight_bytes == 2 * nparam and r.grad_bytes == 4 * nparam
        assert r.p2p_bytes == 2 * s.micro_batch * s.seq * s.hidden      # Eq. (3)
        assert r.workspace_bytes == hh.hh_stage_sizes(cfg, 1, 1)[1]
        assert r.saved_act_bytes > 0
    say("  profile: " + ", ".join("L%d f=%.3fms b=%.3fms" % (r.layer, r.fwd_ms, r.bwd_ms) for r in recs))


def test_trace_counts_launches_per_family_and_honours_the_mask(ctx):
    s = I.LayerShape(512, 4, 128, 1024, 256, 1)
    cfg = L.cfg_of(s, True)
    layer = L.DeviceLayer(I.layer_weights(52, 0, s, True), s, True)
    x_np, dy_np = I.activations(52, s, 0, True)
    x, dy = L.to_dev(x_np, True), L.to_dev(dy_np, True)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    pool_b, wsb = hh.hh_stage_sizes(cfg, 1, 1)
    pool = torch.empty(pool_b, dtype=torch.uint8, device=L.DEV)
    wsp = torch.empty(wsb, dtype=torch.uint8, device=L.DEV)

    def step():
        hh.hh_stage_step(ctx, cfg, [layer.wstruct], [x], [y], [dy], [dx], [layer.gstruct], 1, pool, wsp, L.stream_ptr())

    hh.hh_trace_begin(ctx, 200)
    step()
    step()
    fam = hh.hh_trace_end(ctx)
    f, b = hh.hh_layer_flops(cfg)
    # per layer pass: 4 forward GEMMs, 4 input-gradient GEMMs, 4 weight-gradient GEMMs, one attention each way
    assert [fam[n][0] for n in ("gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd", "attn_bwd")] == [8, 8, 8, 2, 2]
    assert fam["elementwise"][0] > 0 and all(v[1] > 0 for v in fam.values())
    flops = sum(fam[n][2] for n in ("gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd", "attn_bwd"))
    assert abs(flops - 2 * (f + b)) <= 1e-9 * flops
    hh.hh_trace_begin(ctx, 200, ["gemm_tn"])
    step()
    fam = hh.hh_trace_end(ctx)
    assert fam["gemm_tn"][0] == 4 and fam["gemm_tn"][1] > 0
    assert all(v[0] == 0 for n, v in fam.items() if n != "gemm_tn")
    # nothing is recorded once the trace has ended
    step()
    hh.hh_trace_begin(ctx, 1, ["attn_fwd"])
    fam = hh.hh_trace_end(ctx)
    assert all(v[0] == 0 for v in fam.values())


def test_profile_records_feed_the_pipeline_predictor(ctx):
    """Section 3.2: the per-layer times measured on this accelerator (and a second, hypothetical type that is 1.5x
    slower) drive the simulator and the layer split."""
    s = I.LayerShape(512, 4, 128, 1024, 512, 2)
    cfg = L.cfg_of(s, True)
    layer = L.DeviceLayer(I.layer_weights(53, 0, s, True), s, True)
    x_np, dy_np = I.activations(53, s, 0, True)
    x, dy = L.to_dev(x_np, True), L.to_dev(dy_np, True)
    pool_b, wsb = hh.hh_stage_sizes(cfg, 1, 1)
    pool = torch.empty(pool_b, dtype=torch.uint8, device=L.DEV)
    wsp = torch.empty(wsb, dtype=torch.uint8, device=L.DEV)
    rec = hh.hh_layer_profile(ctx, cfg, [layer.wstruct], [layer.gstruct], x, dy, 2, 5, pool, wsp, L.stream_ptr())[0]

    def stage_of(slow):
        return hh.hh_sim_stage(0, 8, rec.fwd_ms * slow, rec.bwd_ms * slow, 2500.0 / slow, 25.0, rec.weight_bytes, rec.grad_bytes,
                               3 * rec.grad_bytes, rec.saved_act_bytes, 0)

    stages = [stage_of(1.0), stage_of(1.0), stage_of(1.5), stage_of(1.5)]
    layers, res = hh.hh_plan_layers(stages, 40, 16, s.micro_batch, s.seq, s.hidden, 1, rec.fwd_flop + rec.bwd_flop)
    assert sum(layers) == 40 and layers[0] > layers[2] and layers[1] > layers[3]
    for st, n in zip(stages, layers):
        st.n_layers = n
    again, fin, peak = hh.hh_sim_pipeline(stages, 16, s.micro_batch, s.seq, s.hidden, 1, rec.fwd_flop + rec.bwd_flop)
    assert again.iter_ms == res.iter_ms and max(fin) == res.iter_ms
    assert peak[0] == layers[0] * (rec.weight_bytes + 4 * rec.grad_bytes) + 4 * layers[0] * rec.saved_act_bytes
    assert 0.0 < res.mfu < 1.0 and res.tokens_per_s_per_device > 0
    say("  planned layers %s, iteration %.2f ms, MFU %.3f of a mean peak of %.0f TFLOP/s" % (layers, res.iter_ms, res.mfu, res.mean_peak_tflops))


# ------------------------------------------------- grouped-query attention
def test_f32_grouped_query_attention(ctx):
    check_layer(ctx, I.LayerShape(128, 4, 64, 96, 70, 2, n_kv_heads=2), False, 71, label="f32-gqa")
    check_layer(ctx, I.LayerShape(128, 4, 64, 96, 33, 1, n_kv_heads=1), False, 72, packed=False, label="f32-mqa-unpacked")


def test_bf16_grouped_query_attention_small_and_long(ctx):
    check_layer(ctx, I.LayerShape(512, 8, 64, 512, 200, 2, n_kv_heads=2), True, 73, label="bf16-gqa-d64")
    check_layer(ctx, I.LayerShape(512, 4, 128, 512, 130, 1, n_kv_heads=1), True, 74, packed=False, label="bf16-mqa-unpacked")
    # long ragged sequence: key tiles split between two wave groups, four query heads per key/value head
    check_layer(ctx, I.LayerShape(1024, 8, 128, 1024, 1500, 1, n_kv_heads=2), True, 75, label="bf16-gqa-long")


def test_bf16_70b_class_tp_share_with_grouped_queries_full_size(ctx):
    # Table 1's 70B / 140B hidden size with the public 64 query / 8 key-value heads at a TP=8 share: 8 local query heads
    # on one local key/value head
    s = I.SHAPE_70B_GQA_TP8
    check_layer(ctx, s, True, 76, label="h8192-gqa-tp8")


@pytest.mark.timeout(900)
def test_bf16_whole_hidden_8192_layer_with_grouped_queries_full_size(ctx):
    # Table 1's hidden size 8192 without tensor parallelism: 64 query heads on 8 key/value heads, ffn 28672 (856 M parameters;
    # the fp32 gradient of the packed gate|up weight is the largest single buffer the GEMM addresses, 1.88 GB)
    check_layer(ctx, I.SHAPE_70B_GQA, True, 77, label="h8192-gqa-tp1")


def test_bf16_grouped_queries_summed_inside_one_workgroup(ctx):
    # enough (key block, key/value head, sample) jobs that each dK/dV workgroup takes both query heads of its group itself
    check_layer(ctx, I.LayerShape(256, 16, 64, 512, 2048, 8, n_kv_heads=8), True, 78, label="gqa-heads-in-one-workgroup")


@pytest.mark.parametrize("seq", [300, 1100])
def test_stage_step_recorded_in_a_graph_replays_bit_identically(ctx, seq):
    # callers may record the stage step into a HIP graph (no allocation, host synchronisation or memset happens inside once
    # the context is warm); every replay, with eager work and synchronisations in between, must give the eager result bit for bit.
    # seq 1100 takes the attention backward through its joint launch (delta kernel, dQ and dK/dV jobs in one grid, partial
    # dK/dV sums of the grouped heads summed and rotated by the reduction kernel); seq 300 through the separate kernels.
    s, k, M = I.LayerShape(512, 8, 64, 768, seq, 2, n_kv_heads=2), 2, 3
    say("[case] graph replay shape=%s k=%d M=%d" % (s, k, M))
    cfg = L.cfg_of(s, True)
    ws_np = [I.layer_weights(91, l, s, True) for l in range(k)]
    acts = [I.activations(91, s, m, True) for m in range(M)]
    layers = [L.DeviceLayer(w, s, True) for w in ws_np]
    xs = [L.to_dev(a[0], True) for a in acts]
    dys = [L.to_dev(a[1], True) for a in acts]
    ys = [torch.empty_like(t) for t in xs]
    dxs = [torch.empty_like(t) for t in xs]
    pool_b, wsb = hh.hh_stage_sizes(cfg, k, M)
    pool = torch.empty(pool_b, dtype=torch.uint8, device=L.DEV)
    wsp = torch.empty(wsb, dtype=torch.uint8, device=L.DEV)
    wst, gst = [l.wstruct for l in layers], [l.gstruct for l in layers]

    def step():
        hh.hh_stage_step(ctx, cfg, wst, xs, ys, dys, dxs, gst, 1, pool, wsp, L.stream_ptr())

    step()
    torch.cuda.synchronize()
    want_y = [t.clone() for t in ys]
    want_dx = [t.clone() for t in dxs]
    want_g = [{n: v.copy() for n, v in l.grads_np().items()} for l in layers]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in ys + dxs:
            t.fill_(float("nan"))
        for l in layers:
            for t in l.g.values():
                t.fill_(7.0)                     # zero_grads_first: the replay must not depend on what the buffers held
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for m in range(M):
            assert torch.equal(ys[m], want_y[m]) and torch.equal(dxs[m], want_dx[m]), (rep, m)
        for l, wg in zip(layers, want_g):
            got = l.grads_np()
            for n in I.WEIGHT_NAMES:
                assert np.array_equal(got[n], wg[n]), (rep, n)
        step()                                   # eager work between replays
        torch.cuda.synchronize()


def test_forward_without_saved_block_and_backward_writing_over_dy(ctx):
    # two conventions of the boundary: saved == NULL runs the forward alone (the workspace then also holds the saved
    # block), and dx may be the buffer dy came in
    s = I.LayerShape(512, 8, 64, 768, 333, 2, n_kv_heads=4)
    say("[case] forward-only and dx aliasing dy, shape=%s" % (s,))
    cfg = L.cfg_of(s, True)
    w = I.layer_weights(93, 0, s, True)
    x_np, dy_np = I.activations(93, s, 0, True)
    layer = L.DeviceLayer(w, s, True)
    y_ref, dx_ref, _ = L.run_layer(ctx, s, True, layer, x_np, dy_np)
    g_ref = {n: v.copy() for n, v in layer.grads_np().items()}
    saved_b, ws_b = hh.hh_layer_sizes(cfg)
    x = L.to_dev(x_np, True)
    y = torch.empty_like(x)
    big_ws = torch.empty(saved_b + ws_b, dtype=torch.uint8, device=L.DEV)
    hh.hh_layer_fwd(ctx, cfg, layer.wstruct, x, y, None, big_ws, L.stream_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(L.to_np(y), y_ref)
    saved = torch.empty(saved_b, dtype=torch.uint8, device=L.DEV)
    ws = torch.empty(ws_b, dtype=torch.uint8, device=L.DEV)
    dy = L.to_dev(dy_np, True)
    hh.hh_layer_fwd(ctx, cfg, layer.wstruct, x, y, saved, ws, L.stream_ptr())
    hh.hh_layer_bwd(ctx, cfg, layer.wstruct, x, saved, dy, dy, layer.gstruct, 0, ws, L.stream_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(L.to_np(dy), dx_ref)
    got = layer.grads_np()
    for n in I.WEIGHT_NAMES:
        assert np.array_equal(got[n], g_ref[n]), n


def test_bf16_seeded_random_small_shapes(ctx):
    # a sweep of small shapes drawn from a fixed seed: ragged sequence lengths around the 64- and 128-row tiles, several
    # samples, both head sizes, grouped and plain heads, packed and separate weights
    rng = np.random.RandomState(20240531)
    for case in range(14):
        d = int(rng.choice([64, 128]))
        nkv = int(rng.choice([1, 2, 3]))
        group = int(rng.choice([1, 1, 2, 4]))
        nh = nkv * group
        hidden = 64 * int(rng.randint(1, 9))
        ffn = 64 * int(rng.randint(1, 9))
        seq = int(rng.choice([1, 2, 31, 63, 64, 65, 127, 128, 129, 191, 257, 300]))
        mb = int(rng.choice([1, 1, 2, 3]))
        s = I.LayerShape(hidden, nh, d, ffn, seq, mb, n_kv_heads=nkv)
        check_layer(ctx, s, True, 300 + case, packed=bool(case % 3), label="random-%d" % case)


def test_fp32_seeded_random_small_shapes(ctx):
    # the fp32 path takes any multiple of 8 for hidden, ffn and n_heads * head_dim
    rng = np.random.RandomState(77)
    for case in range(8):
        d = int(rng.choice([64, 128]))
        nkv = int(rng.choice([1, 2]))
        nh = nkv * int(rng.choice([1, 2, 3]))
        hidden = 8 * int(rng.randint(1, 30))
        ffn = 8 * int(rng.randint(1, 30))
        seq = int(rng.choice([1, 7, 33, 64, 65, 100]))
        mb = int(rng.choice([1, 2, 3]))
        s = I.LayerShape(hidden, nh, d, ffn, seq, mb, n_kv_heads=nkv)
        check_layer(ctx, s, False, 400 + case, packed=bool(case % 2), label="random-f32-%d" % case)


def test_a_recorded_graph_survives_a_later_longer_rotary_table(ctx):
    # a graph recorded at one sequence length keeps the rotary table of that time; a later call with a longer sequence
    # builds a new table and must leave the old one alive for the graph's replays
    s = I.LayerShape(256, 2, 128, 320, 96, 1)
    own = hh.hh_ctx_create(0)
    try:
        cfg = L.cfg_of(s, True)
        layer = L.DeviceLayer(I.layer_weights(95, 0, s, True), s, True)
        x = L.to_dev(I.activations(95, s, 0, True)[0], True)
        y = torch.empty_like(x)
        saved_b, ws_b = hh.hh_layer_sizes(cfg)
        ws = torch.empty(saved_b + ws_b, dtype=torch.uint8, device=L.DEV)
        hh.hh_ctx_reserve(own, cfg)
        hh.hh_layer_fwd(own, cfg, layer.wstruct, x, y, None, ws, L.stream_ptr())
        torch.cuda.synchronize()
        want = y.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                hh.hh_layer_fwd(own, cfg, layer.wstruct, x, y, None, ws, L.stream_ptr())
        torch.cuda.synchronize()
        # a longer sequence on the same context: new table
        s2 = I.LayerShape(256, 2, 128, 320, 700, 1)
        cfg2 = L.cfg_of(s2, True)
        x2 = L.to_dev(I.activations(96, s2, 0, True)[0], True)
        y2 = torch.empty_like(x2)
        sb2, wb2 = hh.hh_layer_sizes(cfg2)
        ws2 = torch.empty(sb2 + wb2, dtype=torch.uint8, device=L.DEV)
        hh.hh_layer_fwd(own, cfg2, layer.wstruct, x2, y2, None, ws2, L.stream_ptr())
        torch.cuda.synchronize()
        for _ in range(2):
            y.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y, want)
    finally:
        torch.cuda.synchronize()
        hh.hh_ctx_destroy(own)
