"""Pins of the CPU oracle against facts that do not come from the oracle itself.

Each test names the part of oracle/decoder_oracle.py it fixes.  A plausible
mistake there (dropped term, wrong sign or index, transposed operand, mask in
the wrong direction) fails at least one of them.  All fp64, CPU only.
"""
import math

import numpy as np
import pytest

from oracle import decoder_oracle as O
from paper_2405_16256_amd import inputs as I


def small_layer(seed=7, H=16, nh=2, d=4, F=24, S=8, B=2, gain_sigma=0.3, wsig=0.4):
    s = I.LayerShape(H, nh, d, F, S, B)
    w = {}
    for p, (n, shp) in enumerate(I.weight_shapes(s).items()):
        if n.startswith("g_"):
            w[n] = I.normal(seed, 100 + p, shp, gain_sigma, 1.0).astype(np.float64)
        else:
            w[n] = I.normal(seed, 100 + p, shp, wsig).astype(np.float64)
    x = I.normal(seed, 1, (B, S, H)).astype(np.float64)
    dy = I.normal(seed, 2, (B, S, H)).astype(np.float64)
    return s, w, x, dy


# ------------------------------------------------------------ P1 brute force
def brute_attention(q, k, v):
    """Pure-Python causal attention written from the definition: for every query
    s only keys t <= s take part; two-pass softmax; no matrices."""
    B, S, nh, d = q.shape
    o = np.zeros_like(q)
    for b in range(B):
        for h in range(nh):
            for s in range(S):
                sc = []
                for t in range(s + 1):
                    acc = 0.0
                    for i in range(d):
                        acc += q[b, s, h, i] * k[b, t, h, i]
                    sc.append(acc / math.sqrt(d))
                mx = max(sc)
                ex = [math.exp(z - mx) for z in sc]
                den = sum(ex)
                for i in range(d):
                    o[b, s, h, i] = sum(ex[t] / den * v[b, t, h, i] for t in range(s + 1))
    return o


def test_attention_matches_brute_force():
    rng = np.random.default_rng(0)
    for (B, S, nh, d) in [(1, 1, 1, 2), (2, 5, 3, 4), (1, 8, 2, 4)]:
        q, k, v = (rng.normal(size=(B, S, nh, d)) * 2 for _ in range(3))
        np.testing.assert_allclose(O.attention_forward(q, k, v), brute_attention(q, k, v),
                                   rtol=1e-12, atol=1e-13)


# ------------------------------------------------- P2 softmax rows / first row
def test_softmax_rows_sum_to_one_and_mask():
    rng = np.random.default_rng(1)
    q, k = rng.normal(size=(33, 8)) * 3, rng.normal(size=(33, 8)) * 3
    P = O.causal_probs(q, k)
    np.testing.assert_allclose(P.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    assert np.all(np.triu(P, 1) == 0.0)        # keys after the query carry no weight
    assert np.all(P[np.tril_indices(33)] > 0.0)
    assert P[0, 0] == 1.0


def test_first_position_outputs_its_own_value():
    rng = np.random.default_rng(2)
    q, k, v = (rng.normal(size=(2, 6, 3, 4)) for _ in range(3))
    o = O.attention_forward(q, k, v)
    assert np.array_equal(o[:, 0], v[:, 0])
    # S = 1: attention is the identity on v
    assert np.array_equal(O.attention_forward(q[:, :1], k[:, :1], v[:, :1]), v[:, :1])


# -------------------------------------------------- P3 finite differences
def _loss(x, w, dy, s):
    y, _ = O.layer_forward(x, w, s.n_heads, s.head_dim, s.rms_eps, s.rope_base)
    return float(np.sum(dy * y))


@pytest.mark.parametrize("cfg", ["small", "cfg1"])
def test_layer_backward_matches_finite_differences(cfg):
    if cfg == "small":
        s, w, x, dy = small_layer()
        ndir = 3
    else:
        s = I.CFG1
        w = {n: a.astype(np.float64) for n, a in I.layer_weights(1001, 0, s, False).items()}
        # larger projection scale than the workload's 0.02 so that every branch
        # contributes visibly to the directional derivative
        for n in w:
            if not n.startswith("g_"):
                w[n] = w[n] * 5.0
        x, dy = (a.astype(np.float64) for a in I.activations(1001, s, 0, False))
        ndir = 1
    y, cache = O.layer_forward(x, w, s.n_heads, s.head_dim, s.rms_eps, s.rope_base)
    dx, g = O.layer_backward(dy, w, cache)
    rng = np.random.default_rng(3)
    targets = [("x", x, dx)] + [(n, w[n], g[n]) for n in I.WEIGHT_NAMES]
    for name, val, grad in targets:
        assert grad.shape == val.shape, name
        for _ in range(ndir):
            dirn = rng.normal(size=val.shape)
            dirn /= np.linalg.norm(dirn)
            eps = 1e-5 * max(1.0, np.linalg.norm(val))

            def at(t):
                if name == "x":
                    return _loss(val + t * dirn, w, dy, s)
                w2 = dict(w)
                w2[name] = val + t * dirn
                return _loss(x, w2, dy, s)
            # 4th-order central difference
            fd = (-at(2 * eps) + 8 * at(eps) - 8 * at(-eps) + at(-2 * eps)) / (12 * eps)
            an = float(np.sum(grad * dirn))
            assert abs(fd - an) <= 2e-7 * max(1.0, abs(an)) + 1e-8, (name, fd, an)


def test_attention_backward_finite_differences_per_operand():
    rng = np.random.default_rng(4)
    q, k, v, do = (rng.normal(size=(1, 7, 2, 4)) for _ in range(4))
    dq, dk, dv = O.attention_backward(do, q, k, v)
    for idx, (val, grad) in enumerate([(q, dq), (k, dk), (v, dv)]):
        dirn = rng.normal(size=val.shape)
        eps = 1e-6

        def at(t):
            ops = [q, k, v]
            ops[idx] = val + t * dirn
            return float(np.sum(do * O.attention_forward(*ops)))
        fd = (at(eps) - at(-eps)) / (2 * eps)
        assert abs(fd - np.sum(grad * dirn)) < 1e-7 * max(1, abs(fd))


# ------------------------------------------------------------- P4 RMSNorm
def test_rmsnorm_value_and_scale_invariance():
    rng = np.random.default_rng(5)
    x = rng.normal(size=(3, 5, 32))
    g = 1 + 0.1 * rng.normal(size=32)
    # direct value: a row of constants c has rms |c| -> output sign(c) * g
    row = np.full((1, 32), -3.0)
    xn, r = O.rmsnorm_forward(row, g, 0.0)
    np.testing.assert_allclose(xn[0], -g, rtol=1e-15)
    np.testing.assert_allclose(r, 1 / 3.0, rtol=1e-15)
    # eps placement: inside the root, added to the mean of squares
    xn, r = O.rmsnorm_forward(row, g, 7.0)
    np.testing.assert_allclose(r, 1 / 4.0, rtol=1e-15)       # sqrt(9 + 7)
    # scale invariance with eps = 0
    a, _ = O.rmsnorm_forward(x, g, 0.0)
    b, _ = O.rmsnorm_forward(2.5 * x, g, 0.0)
    np.testing.assert_allclose(a, b, rtol=1e-13)
    # with eps > 0 the deviation is bounded to first order by eps |1 - c^-2| / (2 mean x^2)
    eps, c = 1e-5, 2.5
    a, _ = O.rmsnorm_forward(x, g, eps)
    b, _ = O.rmsnorm_forward(c * x, g, eps)
    bound = eps * abs(1 - c ** -2) / (2 * np.mean(x * x, axis=-1, keepdims=True))
    assert np.all(np.abs(a - b) <= 1.01 * bound * np.abs(a) + 1e-15)


def test_rmsnorm_backward_euler_identity_and_fd():
    rng = np.random.default_rng(6)
    x = rng.normal(size=(4, 24))
    g = 1 + 0.2 * rng.normal(size=24)
    dxn = rng.normal(size=(4, 24))
    _, r = O.rmsnorm_forward(x, g, 0.0)
    dx, dg = O.rmsnorm_backward(dxn, x, r, g)
    # degree-0 homogeneity (eps = 0)  =>  <x_row, dx_row> = 0
    np.testing.assert_allclose(np.sum(x * dx, axis=-1), 0.0, atol=1e-13)
    # fd with eps > 0
    eps = 1e-3
    _, r = O.rmsnorm_forward(x, g, eps)
    dx, dg = O.rmsnorm_backward(dxn, x, r, g)
    f = lambda xx, gg: float(np.sum(dxn * O.rmsnorm_forward(xx, gg, eps)[0]))
    dirx, dirg = rng.normal(size=x.shape), rng.normal(size=g.shape)
    t = 1e-6
    assert abs((f(x + t * dirx, g) - f(x - t * dirx, g)) / (2 * t) - np.sum(dx * dirx)) < 1e-8
    assert abs((f(x, g + t * dirg) - f(x, g - t * dirg)) / (2 * t) - np.sum(dg * dirg)) < 1e-8


# ---------------------------------------------------------------- P5 RoPE
def test_rope_properties():
    rng = np.random.default_rng(7)
    S, nh, d = 9, 2, 8
    q, k = rng.normal(size=(1, S, nh, d)), rng.normal(size=(1, S, nh, d))
    phi = O.rope_angles(S, d, 10000.0)
    # angle table: phi[s, i] = s * base^(-2i/d)
    assert phi.shape == (S, d // 2)
    assert np.all(phi[0] == 0.0)
    np.testing.assert_allclose(phi[3, 2], 3 * 10000.0 ** (-4 / 8), rtol=1e-15)
    np.testing.assert_allclose(phi[5, 0], 5.0, rtol=1e-15)
    qr, kr = O.rope_forward(q, phi), O.rope_forward(k, phi)
    assert np.array_equal(qr[:, 0], q[:, 0])                       # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(qr, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-13)
    # half-split pairing, explicit 2x2 rotation of channels (i, i + d/2) by +phi
    s_, i_ = 4, 1
    a, b = q[0, s_, 0, i_], q[0, s_, 0, i_ + d // 2]
    ang = s_ * 10000.0 ** (-2 * i_ / d)
    np.testing.assert_allclose(qr[0, s_, 0, i_], a * math.cos(ang) - b * math.sin(ang), rtol=1e-13)
    np.testing.assert_allclose(qr[0, s_, 0, i_ + d // 2], b * math.cos(ang) + a * math.sin(ang), rtol=1e-13)
    # scores depend only on relative position: shift all positions by 5
    phi_shift = phi + 5 * phi[1][None, :]
    q2, k2 = O.rope_forward(q, phi_shift), O.rope_forward(k, phi_shift)
    sc = np.einsum("bshd,bthd->bhst", qr, kr)
    sc2 = np.einsum("bshd,bthd->bhst", q2, k2)
    np.testing.assert_allclose(sc, sc2, atol=1e-12)
    # backward is the inverse rotation (orthogonal map => transpose = inverse)
    np.testing.assert_allclose(O.rope_backward(qr, phi), q, atol=1e-14)
    # and it is the adjoint: <R q, k> = <q, R^T k>
    np.testing.assert_allclose(np.sum(qr * k), np.sum(q * O.rope_backward(k, phi)), rtol=1e-12)


# ---------------------------------------------------------------- P6 SiLU
def test_silu_closed_forms():
    z = np.linspace(-6, 6, 25)
    assert O.silu(np.array(0.0)) == 0.0
    np.testing.assert_allclose(O.silu(z) - O.silu(-z), z, atol=1e-14)
    np.testing.assert_allclose(O.silu(np.array(1.0)), 1 / (1 + math.exp(-1.0)), rtol=1e-15)
    dgt, du = O.swiglu_backward(np.array(1.0), np.array(0.0), np.array(3.0))
    assert dgt == 1.5 and du == 0.0                                  # silu'(0) = 1/2
    # derivative by finite differences
    gt, u, dm = np.array(0.7), np.array(-1.3), np.array(2.0)
    dgt, du = O.swiglu_backward(dm, gt, u)
    t = 1e-6
    np.testing.assert_allclose(dgt, dm * u * (O.silu(gt + t) - O.silu(gt - t)) / (2 * t), rtol=1e-8)
    np.testing.assert_allclose(du, dm * O.silu(gt), rtol=1e-14)


# ------------------------------------------------- P7 zero-weight special cases
def test_zero_output_projections_make_layer_identity():
    s, w, x, dy = small_layer()
    w = dict(w, wo=np.zeros_like(w["wo"]), w_down=np.zeros_like(w["w_down"]))
    y, c = O.layer_forward(x, w, s.n_heads, s.head_dim)
    assert np.array_equal(y, x)
    dx, g = O.layer_backward(dy, w, c)
    assert np.array_equal(dx, dy)
    assert np.any(g["wo"] != 0) and np.any(g["w_down"] != 0)
    for n in ("wq", "wk", "wv", "w_gate", "w_up", "g_attn", "g_mlp"):
        assert np.all(g[n] == 0), n


def test_zero_qk_gives_prefix_mean_of_v():
    s, w, x, dy = small_layer(B=1)
    w = dict(w, wq=np.zeros_like(w["wq"]), wk=np.zeros_like(w["wk"]))
    _, c = O.layer_forward(x, w, s.n_heads, s.head_dim)
    v = c["v"].reshape(1, s.seq, -1)
    prefix_mean = np.cumsum(v, axis=1) / np.arange(1, s.seq + 1)[None, :, None]
    np.testing.assert_allclose(c["a"], prefix_mean, rtol=1e-13, atol=1e-14)


def test_projection_orientation_and_residual_wiring():
    """Weights are [out, in]; with unit gains and eps = 0 the pieces can be recomputed by hand."""
    s, w, x, dy = small_layer(B=1, S=1)
    w = dict(w, g_attn=np.ones(s.hidden), g_mlp=np.ones(s.hidden))
    y, c = O.layer_forward(x, w, s.n_heads, s.head_dim, eps=0.0)
    x0 = x[0, 0]
    xn = x0 / math.sqrt(float(np.mean(x0 ** 2)))
    v = np.array([sum(w["wv"][o, j] * xn[j] for j in range(s.hidden)) for o in range(s.attn)])
    h = x0 + np.array([sum(w["wo"][o, j] * v[j] for j in range(s.attn)) for o in range(s.hidden)])  # S=1: a = v
    hn = h / math.sqrt(float(np.mean(h ** 2)))
    gt = np.array([sum(w["w_gate"][o, j] * hn[j] for j in range(s.hidden)) for o in range(s.ffn)])
    u = np.array([sum(w["w_up"][o, j] * hn[j] for j in range(s.hidden)) for o in range(s.ffn)])
    m = gt / (1 + np.exp(-gt)) * u
    yy = h + np.array([sum(w["w_down"][o, j] * m[j] for j in range(s.ffn)) for o in range(s.hidden)])
    np.testing.assert_allclose(y[0, 0], yy, rtol=1e-12)


# ------------------------------------------------------------ P8 causality
def test_causality_forward_and_backward():
    s, w, x, dy = small_layer(B=1, S=8)
    y, c = O.layer_forward(x, w, s.n_heads, s.head_dim)
    x2 = x.copy()
    x2[0, 5] += 1.0
    y2, _ = O.layer_forward(x2, w, s.n_heads, s.head_dim)
    assert np.array_equal(y[0, :5], y2[0, :5])
    assert np.all(np.any(y[0, 5:] != y2[0, 5:], axis=-1))
    dx, _ = O.layer_backward(dy, w, c)
    dy2 = dy.copy()
    dy2[0, 2] += 1.0
    dx2, _ = O.layer_backward(dy2, w, c)
    # a gradient arriving at position 2 cannot reach inputs at positions > 2
    np.testing.assert_array_equal(dx[0, 3:], dx2[0, 3:])
    assert np.all(np.any(dx[0, :3] != dx2[0, :3], axis=-1))


# ----------------------------------- P9 linearity, batching, head permutation
def test_backward_linear_in_dy_and_batch_duplication():
    s, w, x, dy = small_layer(B=1)
    y, c = O.layer_forward(x, w, s.n_heads, s.head_dim)
    dx1, g1 = O.layer_backward(dy, w, c)
    dx3, g3 = O.layer_backward(3.0 * dy, w, c)
    np.testing.assert_allclose(dx3, 3 * dx1, rtol=1e-12)
    np.testing.assert_allclose(g3["wq"], 3 * g1["wq"], rtol=1e-12, atol=1e-14)
    xx, dd = np.concatenate([x, x]), np.concatenate([dy, dy])
    y2, c2 = O.layer_forward(xx, w, s.n_heads, s.head_dim)
    assert np.array_equal(y2[0], y2[1]) and np.array_equal(y2[0], y[0])
    dx2, g2 = O.layer_backward(dd, w, c2)
    for n in I.WEIGHT_NAMES:
        np.testing.assert_allclose(g2[n], 2 * g1[n], rtol=1e-12, atol=1e-14)


def test_head_permutation_leaves_output_unchanged():
    s, w, x, dy = small_layer(nh=3, H=12, d=4)
    d = s.head_dim
    perm = np.array([2, 0, 1])
    cols = (perm[:, None] * d + np.arange(d)[None, :]).reshape(-1)
    w2 = dict(w, wq=w["wq"][cols], wk=w["wk"][cols], wv=w["wv"][cols], wo=w["wo"][:, cols])
    y, _ = O.layer_forward(x, w, s.n_heads, d)
    y2, _ = O.layer_forward(x, w2, s.n_heads, d)
    np.testing.assert_allclose(y, y2, rtol=1e-12, atol=1e-13)


# ------------------------------------------------- P10 stage composition
def test_stage_step_equals_hand_chained_layers_and_accumulates():
    s, w0, x0, dy0 = small_layer(seed=11)
    _, w1, x1, dy1 = small_layer(seed=12)
    ws = [w0, w1]
    ys, dxs, grads = O.stage_step([x0, x1], [dy0, dy1], ws, s.n_heads, s.head_dim)
    tot = [dict((n, 0.0) for n in I.WEIGHT_NAMES) for _ in ws]
    for m, (x, dy) in enumerate([(x0, dy0), (x1, dy1)]):
        h1, c0 = O.layer_forward(x, w0, s.n_heads, s.head_dim)
        y, c1 = O.layer_forward(h1, w1, s.n_heads, s.head_dim)
        d1, g1 = O.layer_backward(dy, w1, c1)
        d0, g0 = O.layer_backward(d1, w0, c0)
        assert np.array_equal(ys[m], y) and np.array_equal(dxs[m], d0)
        for n in I.WEIGHT_NAMES:
            tot[0][n] = tot[0][n] + g0[n]
            tot[1][n] = tot[1][n] + g1[n]
    for l in range(2):
        for n in I.WEIGHT_NAMES:
            np.testing.assert_allclose(grads[l][n], tot[l][n], rtol=1e-13, atol=1e-15)
    # M identical micro-batches => M x the gradient of one
    _, _, g3 = O.stage_step([x0] * 3, [dy0] * 3, ws, s.n_heads, s.head_dim)
    _, _, g1 = O.stage_step([x0], [dy0], ws, s.n_heads, s.head_dim)
    for n in I.WEIGHT_NAMES:
        np.testing.assert_allclose(g3[0][n], 3 * g1[0][n], rtol=1e-12, atol=1e-14)


def test_stage_finite_difference_through_two_layers():
    s, w0, x, dy = small_layer(seed=21, B=1)
    _, w1, _, _ = small_layer(seed=22, B=1)
    ys, dxs, grads = O.stage_step([x], [dy], [w0, w1], s.n_heads, s.head_dim)
    rng = np.random.default_rng(8)
    dirn = rng.normal(size=w0["w_up"].shape)
    t = 1e-6

    def at(e):
        wa = dict(w0, w_up=w0["w_up"] + e * dirn)
        yy, _, _ = O.stage_step([x], [dy], [wa, w1], s.n_heads, s.head_dim)
        return float(np.sum(dy * yy[0]))
    fd = (at(t) - at(-t)) / (2 * t)
    assert abs(fd - np.sum(grads[0]["w_up"] * dirn)) < 1e-7 * max(1, abs(fd))


# ------------------------------------------- P11 autograd third opinion
def test_against_autograd_of_the_same_equations():
    torch = pytest.importorskip("torch")
    s, w, x, dy = small_layer(H=32, nh=2, d=8, F=40, S=12, B=2)
    tw = {n: torch.tensor(a, dtype=torch.float64, requires_grad=True) for n, a in w.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    B, S, H = x.shape
    nh, d = s.n_heads, s.head_dim

    def norm(t, g):
        return t * torch.rsqrt(t.pow(2).mean(-1, keepdim=True) + s.rms_eps) * g

    def rope(t):
        pos = torch.arange(S, dtype=torch.float64)
        inv = s.rope_base ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
        ang = torch.outer(pos, inv)
        cos = torch.cat([ang.cos(), ang.cos()], -1)[None, :, None, :]
        sin = torch.cat([ang.sin(), ang.sin()], -1)[None, :, None, :]
        rot = torch.cat([-t[..., d // 2:], t[..., :d // 2]], -1)
        return t * cos + rot * sin

    xn = norm(tx, tw["g_attn"])
    q = rope(torch.nn.functional.linear(xn, tw["wq"]).view(B, S, nh, d)).transpose(1, 2)
    k = rope(torch.nn.functional.linear(xn, tw["wk"]).view(B, S, nh, d)).transpose(1, 2)
    v = torch.nn.functional.linear(xn, tw["wv"]).view(B, S, nh, d).transpose(1, 2)
    a = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
    a = a.transpose(1, 2).reshape(B, S, nh * d)
    h = tx + torch.nn.functional.linear(a, tw["wo"])
    hn = norm(h, tw["g_mlp"])
    m = torch.nn.functional.silu(torch.nn.functional.linear(hn, tw["w_gate"])) * \
        torch.nn.functional.linear(hn, tw["w_up"])
    y = h + torch.nn.functional.linear(m, tw["w_down"])
    y.backward(torch.tensor(dy))

    yo, c = O.layer_forward(x, w, nh, d, s.rms_eps, s.rope_base)
    dxo, g = O.layer_backward(dy, w, c)
    np.testing.assert_allclose(yo, y.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dxo, tx.grad.numpy(), rtol=1e-10, atol=1e-11)
    for n in I.WEIGHT_NAMES:
        np.testing.assert_allclose(g[n], tw[n].grad.numpy(), rtol=1e-10, atol=1e-11, err_msg=n)


# ------------------------------------------------------ grouped-query attention
def test_grouped_query_attention_equals_multi_head_with_repeated_kv_heads():
    """With key/value heads shared by G query heads the layer must equal the multi-head layer whose wk, wv rows are
    the shared heads repeated G times, and the gradient of a shared head is the sum over its copies."""
    H, nh, nkv, d, F, S, B = 24, 6, 2, 4, 20, 7, 2
    G = nh // nkv
    s = I.LayerShape(H, nh, d, F, S, B, n_kv_heads=nkv)
    w = {n: I.normal(11, 200 + p, shp, 0.4, 1.0 if n.startswith("g_") else 0.0).astype(np.float64)
         for p, (n, shp) in enumerate(I.weight_shapes(s).items())}
    assert w["wk"].shape == (nkv * d, H) and w["wq"].shape == (nh * d, H)
    x = I.normal(11, 1, (B, S, H)).astype(np.float64)
    dy = I.normal(11, 2, (B, S, H)).astype(np.float64)
    y, cache = O.layer_forward(x, w, nh, d, n_kv_heads=nkv)
    dx, g = O.layer_backward(dy, w, cache)
    rep = lambda m: m.reshape(nkv, 1, d, H).repeat(G, axis=1).reshape(nh * d, H)
    w2 = dict(w, wk=rep(w["wk"]), wv=rep(w["wv"]))
    y2, cache2 = O.layer_forward(x, w2, nh, d)
    dx2, g2 = O.layer_backward(dy, w2, cache2)
    np.testing.assert_allclose(y, y2, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dx, dx2, rtol=1e-11, atol=1e-12)
    fold = lambda m: m.reshape(nkv, G, d, H).sum(axis=1).reshape(nkv * d, H)
    np.testing.assert_allclose(g["wk"], fold(g2["wk"]), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(g["wv"], fold(g2["wv"]), rtol=1e-11, atol=1e-12)
    for n in ("wq", "wo", "g_attn", "g_mlp", "w_gate", "w_up", "w_down"):
        np.testing.assert_allclose(g[n], g2[n], rtol=1e-11, atol=1e-12)
    # the grouping is by consecutive query heads: pairing head h with kv head h % nkv instead must differ
    q = cache["qr"]
    wrong = np.stack([O.causal_probs(q[0, :, h], cache["kr"][0, :, h % nkv]) @ cache["v"][0, :, h % nkv] for h in range(nh)], axis=1)
    assert np.abs(wrong.reshape(S, nh * d) - cache["a"][0]).max() > 1e-3


def test_grouped_query_layer_finite_differences():
    H, nh, nkv, d, F, S, B = 12, 4, 1, 4, 10, 5, 1
    s = I.LayerShape(H, nh, d, F, S, B, n_kv_heads=nkv)
    w = {n: I.normal(12, 300 + p, shp, 0.4, 1.0 if n.startswith("g_") else 0.0).astype(np.float64)
         for p, (n, shp) in enumerate(I.weight_shapes(s).items())}
    x = I.normal(12, 1, (B, S, H)).astype(np.float64)
    dy = I.normal(12, 2, (B, S, H)).astype(np.float64)
    y, cache = O.layer_forward(x, w, nh, d, n_kv_heads=nkv)
    dx, g = O.layer_backward(dy, w, cache)
    loss = lambda xx, ww: float(np.sum(O.layer_forward(xx, ww, nh, d, n_kv_heads=nkv)[0] * dy))
    rng = np.random.default_rng(3)
    eps = 1e-4
    for name in ("wk", "wv", "wq", None):
        arr = x if name is None else w[name]
        grad = dx if name is None else g[name]
        for _ in range(6):
            idx = tuple(rng.integers(0, n) for n in arr.shape)
            def at(delta):
                a2 = arr.copy(); a2[idx] += delta
                return loss(a2, w) if name is None else loss(x, dict(w, **{name: a2}))
            fd = (-at(2 * eps) + 8 * at(eps) - 8 * at(-eps) + at(-2 * eps)) / (12 * eps)
            assert abs(fd - grad[idx]) <= 1e-7 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])
