"""CPU fp64 oracle for the decoder-stage step.  TEST INFRASTRUCTURE ONLY.

This file defines what the GPU library must compute; it is never part of the
product path.  Only tests/, the smoke check and the benchmark's cpu_baseline
leg may import it.  It shares no code with the HIP kernels and imports nothing
from the package.

What is computed.  The paper trains Llama2 models (Section 4.2, "Model and
Dataset"; Table 1 gives layer counts and hidden sizes) and assigns each
device a pipeline stage of 1..k consecutive layers that processes the batch as
micro-batches (Section 2.3).  The paper does not restate the layer, so the
oracle writes out the standard pre-norm Llama decoder layer: RMSNorm ->
Q/K/V projections -> rotary embedding (half-split pairing) -> causal softmax
attention -> output projection + residual -> RMSNorm -> SwiGLU MLP + residual,
with no biases and no dropout, and its exact reverse-mode derivative.  The
result is a plain mathematical definition, so the oracle is that definition
typed out in fp64: full S x S score matrices, no tiling, no fusion, no
re-ordering.  `numpy.matmul` is the only library primitive used as a step.

Conventions: activations [B, S, feat]; weights [out, in]; head h owns columns
h*d .. h*d+d-1 of q, k, v; positions start at 0; gradients of parameters are
summed over all tokens of all samples and (in `stage_step`) over micro-batches
(plain sum, no 1/M).

Pins (tests/test_oracle_pins.py): brute-force attention on tiny inputs, softmax
row sums, finite differences of the whole layer and stage, RMSNorm scale
invariance and Euler identity, RoPE isometry / shift invariance, SiLU closed
forms, zero-weight special cases, causality, linearity, head permutation,
stage composition, and an autograd cross-check.  No function here is
"parity unpinned".
"""
import numpy as np

F64 = np.float64


# ------------------------------------------------------------------ RMSNorm
def rmsnorm_forward(x, g, eps):
    """r[s] = 1/sqrt(mean_j x[s,j]^2 + eps);  xn = x * r * g.   x: [..., H]."""
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x * r * g, r


def rmsnorm_backward(dxn, x, r, g):
    """Gradient of xn = x*r*g wrt x and g (rows independent).

    With u = x*r (the normalised row) and w = dxn*g:
      dg[j] = sum_rows dxn[.,j] u[.,j]
      dx    = r * (w - u * mean_j(w_j u_j))
    """
    u = x * r
    w = dxn * g
    dg = np.sum((dxn * u).reshape(-1, x.shape[-1]), axis=0)
    dx = r * (w - u * np.mean(w * u, axis=-1, keepdims=True))
    return dx, dg


# --------------------------------------------------------------------- RoPE
def rope_angles(seq, head_dim, base):
    """phi[s, i] = s * base^(-2i/d), i in [0, d/2)."""
    i = np.arange(head_dim // 2, dtype=F64)
    theta = base ** (-2.0 * i / head_dim)
    return np.arange(seq, dtype=F64)[:, None] * theta[None, :]


def rope_forward(t, phi):
    """Rotate channel pairs (i, i+d/2) of t[B,S,nh,d] by +phi[s,i]."""
    half = t.shape[-1] // 2
    c = np.cos(phi)[None, :, None, :]
    s = np.sin(phi)[None, :, None, :]
    a, b = t[..., :half], t[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def rope_backward(dt, phi):
    """Transpose of the rotation = rotation by -phi."""
    half = dt.shape[-1] // 2
    c = np.cos(phi)[None, :, None, :]
    s = np.sin(phi)[None, :, None, :]
    a, b = dt[..., :half], dt[..., half:]
    return np.concatenate([a * c + b * s, b * c - a * s], axis=-1)


# ---------------------------------------------------------------- attention
def causal_probs(qh, kh):
    """P[s,t] = softmax over t<=s of qh[s].kh[t]/sqrt(d); 0 for t>s.  qh,kh: [S,d]."""
    S, d = qh.shape
    z = (qh @ kh.T) / np.sqrt(F64(d))
    keep = np.tril(np.ones((S, S), dtype=bool))
    z = np.where(keep, z, -np.inf)
    z = z - np.max(z, axis=1, keepdims=True)
    e = np.exp(z)                      # exp(-inf) = 0 for the excluded keys
    return e / np.sum(e, axis=1, keepdims=True)


def attention_forward(q, k, v):
    """q: [B,S,nh,d]; k,v: [B,S,nkv,d] with nh a multiple of nkv -> o [B,S,nh,d].  One causal softmax per
    (sample, query head); query head h reads key/value head h // (nh // nkv) (grouped-query attention;
    nkv == nh is the ordinary multi-head case)."""
    B, S, nh, d = q.shape
    G = nh // k.shape[2]
    o = np.empty_like(q)
    for b in range(B):
        for h in range(nh):
            P = causal_probs(q[b, :, h], k[b, :, h // G])
            o[b, :, h] = P @ v[b, :, h // G]
    return o


def attention_backward(do, q, k, v):
    """Gradients of attention_forward wrt q, k, v; a key/value head collects the gradients of its G query heads."""
    B, S, nh, d = q.shape
    G = nh // k.shape[2]
    dq, dk, dv = np.empty_like(q), np.zeros_like(k), np.zeros_like(v)
    inv = 1.0 / np.sqrt(F64(d))
    for b in range(B):
        for h in range(nh):
            qh, kh, vh, doh = q[b, :, h], k[b, :, h // G], v[b, :, h // G], do[b, :, h]
            P = causal_probs(qh, kh)
            dv[b, :, h // G] += P.T @ doh
            dP = doh @ vh.T
            D = np.sum(P * dP, axis=1, keepdims=True)
            dZ = P * (dP - D)
            dq[b, :, h] = (dZ @ kh) * inv
            dk[b, :, h // G] += (dZ.T @ qh) * inv
    return dq, dk, dv


# ------------------------------------------------------------------- SwiGLU
def silu(z):
    return z / (1.0 + np.exp(-z))


def swiglu_backward(dm, gt, u):
    """m = silu(gt)*u  ->  (d gt, d u)."""
    sg = 1.0 / (1.0 + np.exp(-gt))
    dgt = dm * u * sg * (1.0 + gt * (1.0 - sg))
    du = dm * gt * sg
    return dgt, du


# ------------------------------------------------------------ decoder layer
def _f64(w):
    return {n: np.asarray(a, dtype=F64) for n, a in w.items()}


def layer_forward(x, w, n_heads, head_dim, eps=1e-5, rope_base=10000.0, n_kv_heads=None):
    """One decoder layer.  x: [B,S,H];  w: dict of the 9 parameters (wk, wv: [n_kv_heads*head_dim, H]).
    -> (y, cache)."""
    x = np.asarray(x, dtype=F64)
    w = _f64(w)
    B, S, H = x.shape
    nh, d = n_heads, head_dim
    nkv = nh if n_kv_heads is None else n_kv_heads
    phi = rope_angles(S, d, rope_base)

    xn, r1 = rmsnorm_forward(x, w["g_attn"], eps)
    q = (xn @ w["wq"].T).reshape(B, S, nh, d)
    k = (xn @ w["wk"].T).reshape(B, S, nkv, d)
    v = (xn @ w["wv"].T).reshape(B, S, nkv, d)
    qr = rope_forward(q, phi)
    kr = rope_forward(k, phi)
    o = attention_forward(qr, kr, v)
    a = o.reshape(B, S, nh * d)
    h = x + a @ w["wo"].T

    hn, r2 = rmsnorm_forward(h, w["g_mlp"], eps)
    gt = hn @ w["w_gate"].T
    u = hn @ w["w_up"].T
    m = silu(gt) * u
    y = h + m @ w["w_down"].T

    cache = dict(x=x, r1=r1, xn=xn, qr=qr, kr=kr, v=v, a=a, h=h, r2=r2, hn=hn,
                 gt=gt, u=u, m=m, phi=phi, nh=nh, nkv=nkv, d=d)
    return y, cache


def layer_backward(dy, w, cache):
    """Reverse pass of layer_forward.  -> (dx, grads dict with the 9 parameter names)."""
    dy = np.asarray(dy, dtype=F64)
    w = _f64(w)
    c = cache
    B, S, H = dy.shape
    nh, nkv, d = c["nh"], c["nkv"], c["d"]
    T = B * S
    flat = lambda t: t.reshape(T, -1)
    g = {}

    # y = h + m Wd^T
    g["w_down"] = flat(dy).T @ flat(c["m"])
    dm = dy @ w["w_down"]
    dgt, du = swiglu_backward(dm, c["gt"], c["u"])
    g["w_gate"] = flat(dgt).T @ flat(c["hn"])
    g["w_up"] = flat(du).T @ flat(c["hn"])
    dhn = dgt @ w["w_gate"] + du @ w["w_up"]
    dh_norm, g["g_mlp"] = rmsnorm_backward(dhn, c["h"], c["r2"], w["g_mlp"])
    dh = dy + dh_norm

    # h = x + a Wo^T
    g["wo"] = flat(dh).T @ flat(c["a"])
    do = (dh @ w["wo"]).reshape(B, S, nh, d)
    dqr, dkr, dv = attention_backward(do, c["qr"], c["kr"], c["v"])
    dq = rope_backward(dqr, c["phi"]).reshape(B, S, nh * d)
    dk = rope_backward(dkr, c["phi"]).reshape(B, S, nkv * d)
    dv = dv.reshape(B, S, nkv * d)
    g["wq"] = flat(dq).T @ flat(c["xn"])
    g["wk"] = flat(dk).T @ flat(c["xn"])
    g["wv"] = flat(dv).T @ flat(c["xn"])
    dxn = dq @ w["wq"] + dk @ w["wk"] + dv @ w["wv"]
    dx_norm, g["g_attn"] = rmsnorm_backward(dxn, c["x"], c["r1"], w["g_attn"])
    dx = dh + dx_norm
    return dx, g


# --------------------------------------------------------------- stage step
def stage_step(xs, dys, ws, n_heads, head_dim, eps=1e-5, rope_base=10000.0, n_kv_heads=None):
    """A pipeline stage of k = len(ws) layers over M = len(xs) micro-batches.

    All micro-batches run forward through the k layers (layer l's output feeds
    layer l+1), then all run backward through the layers in reverse; parameter
    gradients are summed over micro-batches.  -> (ys, dxs, grads[l][name]).
    """
    k, M = len(ws), len(xs)
    caches, ys = [], []
    for m in range(M):
        t, cs = np.asarray(xs[m], dtype=F64), []
        for l in range(k):
            t, c = layer_forward(t, ws[l], n_heads, head_dim, eps, rope_base, n_kv_heads)
            cs.append(c)
        ys.append(t)
        caches.append(cs)
    grads = [None] * k
    dxs = []
    for m in range(M):
        dt = np.asarray(dys[m], dtype=F64)
        for l in reversed(range(k)):
            dt, g = layer_backward(dt, ws[l], caches[m][l])
            if grads[l] is None:
                grads[l] = g
            else:
                for n in g:
                    grads[l][n] = grads[l][n] + g[n]
        dxs.append(dt)
    return ys, dxs, grads
