"""Where the bf16 path's 1-2e-2 error at hidden 12288 comes from.  No GPU: the layer equations of the oracle are
evaluated in fp64 with a round-to-nearest-even bf16 rounding applied ONLY at the tensors the GPU path stores in bf16
(normalised activations, rotated q and k, v, the attention output, the residual stream, gate, up, m, the probabilities
and score gradients that feed the matrix cores, and the gradient tensors passed between kernels); every sum stays
exact.  The error of that evaluation against the exact one is the floor any bf16-storage implementation has, and it
grows with the hidden size because the attention scores of N(0, 0.02^2) projections of a 12288-wide normalised row
have a standard deviation near 5: a 2^-9 relative rounding of q and k moves the scores by about 0.01 absolute, i.e. the
softmax weights by about 1 %."""
import numpy as np

from oracle import decoder_oracle as O
from paper_2405_16256_amd import inputs as I


def bf(a):
    return I.round_to_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64)


def rel(a, b):
    return float(np.linalg.norm((a - b).ravel()) / np.linalg.norm(b.ravel()))


def rounded_layer(x, dy, w, s):
    """Forward and backward of the decoder layer with bf16 storage rounding and exact arithmetic in between."""
    B, S, H = x.shape
    nh, d = s.n_heads, s.head_dim
    w = {n: np.asarray(a, dtype=np.float64) for n, a in w.items()}
    phi = O.rope_angles(S, d, s.rope_base)
    xn, r1 = O.rmsnorm_forward(x, w["g_attn"], s.rms_eps)
    xn = bf(xn)
    q = O.rope_forward(bf(xn @ w["wq"].T).reshape(B, S, nh, d), phi)
    k = O.rope_forward(bf(xn @ w["wk"].T).reshape(B, S, nh, d), phi)
    q, k, v = bf(q), bf(k), bf(xn @ w["wv"].T).reshape(B, S, nh, d)
    o = np.empty_like(q)
    P = {}
    for b in range(B):
        for h in range(nh):
            p = O.causal_probs(q[b, :, h], k[b, :, h])
            P[b, h] = p
            # the matrix cores see rounded unnormalised weights; the normaliser is the sum of the unrounded ones
            scale = np.max(p, axis=1, keepdims=True)
            o[b, :, h] = (bf(p / scale) @ v[b, :, h]) * scale
    a = bf(o.reshape(B, S, nh * d))
    h_ = bf(x + a @ w["wo"].T)
    hn, r2 = O.rmsnorm_forward(h_, w["g_mlp"], s.rms_eps)
    hn = bf(hn)
    gt, u = bf(hn @ w["w_gate"].T), bf(hn @ w["w_up"].T)
    m = bf(O.silu(gt) * u)
    y = bf(h_ + m @ w["w_down"].T)
    # backward
    flat = lambda t: t.reshape(B * S, -1)
    g = {}
    g["w_down"] = flat(dy).T @ flat(m)
    dm = bf(dy @ w["w_down"])
    dgt, du = O.swiglu_backward(dm, gt, u)
    dgt, du = bf(dgt), bf(du)
    g["w_gate"], g["w_up"] = flat(dgt).T @ flat(hn), flat(du).T @ flat(hn)
    dhn = bf(dgt @ w["w_gate"] + du @ w["w_up"])
    dh_norm, g["g_mlp"] = O.rmsnorm_backward(dhn, h_, r2, w["g_mlp"])
    dh = bf(dy + dh_norm)
    g["wo"] = flat(dh).T @ flat(a)
    do = bf(dh @ w["wo"]).reshape(B, S, nh, d)
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    inv = 1.0 / np.sqrt(float(d))
    for b in range(B):
        for h in range(nh):
            p, doh = P[b, h], do[b, :, h]
            dv[b, :, h] = bf(p).T @ doh
            dP = doh @ v[b, :, h].T
            D = np.sum(doh * a.reshape(B, S, nh, d)[b, :, h], axis=1, keepdims=True)      # <dO, O> of the stored output
            dZ = bf(p * (dP - D))
            dq[b, :, h] = (dZ @ k[b, :, h]) * inv
            dk[b, :, h] = (dZ.T @ q[b, :, h]) * inv
    dq = bf(O.rope_backward(bf(dq), phi)).reshape(B, S, nh * d)
    dk = bf(O.rope_backward(bf(dk), phi)).reshape(B, S, nh * d)
    dv = bf(dv).reshape(B, S, nh * d)
    g["wq"], g["wk"], g["wv"] = flat(dq).T @ flat(xn), flat(dk).T @ flat(xn), flat(dv).T @ flat(xn)
    dxn = bf(dq @ w["wq"] + dk @ w["wk"] + dv @ w["wv"])
    dx_norm, g["g_attn"] = O.rmsnorm_backward(dxn, x, r1, w["g_attn"])
    return y, bf(dh + dx_norm), g


def floor_errors(hidden, seed):
    s = I.LayerShape(hidden, 2, 128, 256, 192, 1)
    w = I.layer_weights(seed, 0, s, True)
    x, dy = I.activations(seed, s, 0, True)
    yo, cache = O.layer_forward(x, w, s.n_heads, s.head_dim, s.rms_eps, s.rope_base)
    dxo, go = O.layer_backward(dy, w, cache)
    y, dx, g = rounded_layer(x.astype(np.float64), dy.astype(np.float64), w, s)
    e = {"y": rel(y, yo), "dx": rel(dx, dxo)}
    e.update({"d" + n: rel(g[n], go[n]) for n in I.WEIGHT_NAMES})
    qr = cache["qr"][0, :, 0]
    kr = cache["kr"][0, :, 0]
    score_std = float(np.std((qr @ kr.T)[np.tril_indices(s.seq)] / np.sqrt(128.0)))
    return e, score_std


def test_storage_rounding_alone_gives_the_error_level_seen_at_hidden_12288():
    wide, std_wide = floor_errors(12288, 901)
    narrow, std_narrow = floor_errors(1024, 902)
    print("hidden 12288: score std %.2f" % std_wide, {k: "%.2e" % v for k, v in wide.items()})
    print("hidden  1024: score std %.2f" % std_narrow, {k: "%.2e" % v for k, v in narrow.items()})
    # N(0, 0.02^2) projections of a unit-RMS row: q, k entries ~ 0.02 sqrt(H), scores ~ 0.02^2 H sqrt(128) / sqrt(128)... = 4e-4 H
    assert 4.0 < std_wide < 6.0 and std_narrow < 0.6
    # the floor at the measured width is the 1-2e-2 the GPU shows there (y 1.2e-2, dx 1.8e-2, dwq 1.9e-2), inside the tolerances
    assert 5e-3 < wide["y"] < 2e-2
    assert 8e-3 < wide["dwq"] < 5e-2 and 8e-3 < wide["dx"] < 5e-2
    # and it is the score magnitude that lifts it: the same evaluation at hidden 1024 stays at a few 1e-3
    assert narrow["y"] < 6e-3 and narrow["dwq"] < 8e-3
    assert wide["dwq"] > 1.8 * narrow["dwq"] and wide["y"] > 1.5 * narrow["y"]
