"""Seeded synthetic inputs for Llama-style decoder layers.

This module only *draws numbers*: it holds no arithmetic of the decoder layer.
It is the one piece of code that both the GPU path's tests and the CPU oracle's
tests consume, so that both see bit-identical inputs.

Generator (counter based, stateless): element ``i`` of tensor ``tid`` under
``seed`` is

    key = mix64(mix64(seed) + tid)
    u1  = ((mix64(key + 2 i)     >> 11) + 1) * 2**-53        in (0, 1]
    u2  =  (mix64(key + 2 i + 1) >> 11)      * 2**-53        in [0, 1)
    z   = sqrt(-2 ln u1) * cos(2 pi u2)                      ~ N(0, 1)

with ``mix64`` the splitmix64 output finaliser (Steele, Lea, Flood 2014).  The
value is ``mean + scale * z`` evaluated in fp64 and cast to fp32.

Distributions follow the workload description of the decoder-stage step: the
projection matrices are N(0, 0.02^2), the RMSNorm gains are 1 + 0.02 N(0, 1)
(a gain drawn around zero would shrink every branch to nothing and let the
residual hide errors), activations and upstream gradients are N(0, 1).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK = (1 << 64) - 1

# Tensor ids.  x and dy of micro-batch m use  TID_X + (m << 32), TID_DY + (m << 32);
# parameter p of layer l uses  TID_W0 + 16 * l + p  with p indexing WEIGHT_NAMES.
TID_X = 0
TID_DY = 1
TID_W0 = 10
WEIGHT_NAMES = ("g_attn", "wq", "wk", "wv", "wo", "g_mlp", "w_gate", "w_up", "w_down")


def _mix64_int(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _normal_chunk(out: np.ndarray, key: int, lo: int, hi: int, scale: float, mean: float) -> None:
    two53 = 2.0 ** -53
    with np.errstate(over="ignore"):
        c = np.arange(2 * lo, 2 * hi, 2, dtype=np.uint64) + np.uint64(key)
        u1 = ((_mix64(c) >> np.uint64(11)).astype(np.float64) + 1.0) * two53
        u2 = (_mix64(c + np.uint64(1)) >> np.uint64(11)).astype(np.float64) * two53
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[lo:hi] = (mean + scale * z).astype(np.float32)


def normal(seed: int, tid: int, shape, scale: float = 1.0, mean: float = 0.0,
           chunk: int = 1 << 20) -> np.ndarray:
    """fp32 array of ``shape`` with entries mean + scale * N(0,1); see module doc.
    Elements are independent of the chunking (large draws are filled by a few threads)."""
    n = int(np.prod(shape)) if len(tuple(shape)) else 1
    out = np.empty(n, dtype=np.float32)
    key = _mix64_int(_mix64_int(seed) + tid)
    spans = [(lo, min(n, lo + chunk)) for lo in range(0, n, chunk)]
    if len(spans) <= 2:
        for lo, hi in spans:
            _normal_chunk(out, key, lo, hi, scale, mean)
    else:
        nthreads = max(1, min(16, os.cpu_count() or 1))
        with ThreadPoolExecutor(nthreads) as ex:
            list(ex.map(lambda sp: _normal_chunk(out, key, sp[0], sp[1], scale, mean), spans))
    return out.reshape(shape)


# ---------------------------------------------------------------- bf16 storage
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 values that are exactly representable in bf16 (RNE)."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


# ---------------------------------------------------------------- layer inputs
@dataclass(frozen=True)
class LayerShape:
    hidden: int
    n_heads: int
    head_dim: int
    ffn: int
    seq: int
    micro_batch: int = 1
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    n_kv_heads: int = 0          # 0: as many as n_heads (multi-head attention); else a divisor of n_heads

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads or self.n_heads

    @property
    def attn(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def attn_kv(self) -> int:
        return self.kv_heads * self.head_dim

    @property
    def tokens(self) -> int:
        return self.seq * self.micro_batch


# The five workload shapes (dtype, shape, layers k, micro-batches M, seed).
CFG1 = LayerShape(256, 4, 64, 688, 128, 1)          # tiny, fp32
CFG2 = LayerShape(4096, 32, 128, 11008, 2048, 1)    # 7B-class layer, bf16
CFG3 = LayerShape(12288, 12, 128, 4096, 4096, 1)    # 140B-class layer at a TP=8 share, bf16
# further Table 1 model classes (hidden size from the table; head count and FFN width are the public
# Llama-2 values for that hidden size, which the paper does not state)
SHAPE_13B = LayerShape(5120, 40, 128, 13824, 2048, 1)        # 13B-class layer: 40 x 128 heads
SHAPE_70B_TP8 = LayerShape(8192, 8, 128, 3584, 4096, 1)      # 70B/140B-class hidden 8192 at a TP=8 share (MHA)
SHAPE_70B_GQA_TP8 = LayerShape(8192, 8, 128, 3584, 4096, 1, n_kv_heads=1)   # same, 64 query / 8 key-value heads over TP=8
SHAPE_70B_GQA = LayerShape(8192, 64, 128, 28672, 4096, 1, n_kv_heads=8)        # the whole hidden-8192 layer (no tensor parallelism)
SEEDS = {"cfg1": 1001, "cfg2": 1002, "cfg3": 1003, "cfg4": 1004, "cfg5": 1005}


def weight_shapes(s: LayerShape) -> dict:
    H, A, Akv, F = s.hidden, s.attn, s.attn_kv, s.ffn
    return {"g_attn": (H,), "wq": (A, H), "wk": (Akv, H), "wv": (Akv, H), "wo": (H, A),
            "g_mlp": (H,), "w_gate": (F, H), "w_up": (F, H), "w_down": (H, F)}


def layer_weights(seed: int, layer: int, s: LayerShape, bf16: bool) -> dict:
    """fp32 arrays (bf16-representable when ``bf16``) for the 9 parameters of one layer."""
    out = {}
    for p, (name, shp) in enumerate(weight_shapes(s).items()):
        tid = TID_W0 + 16 * layer + p
        if name.startswith("g_"):
            w = normal(seed, tid, shp, scale=0.02, mean=1.0)
        else:
            w = normal(seed, tid, shp, scale=0.02)
        out[name] = round_to_bf16(w) if bf16 else w
    return out


def activations(seed: int, s: LayerShape, micro: int, bf16: bool):
    """(x, dy), each [micro_batch, seq, hidden] fp32 (bf16-representable when ``bf16``)."""
    shp = (s.micro_batch, s.seq, s.hidden)
    x = normal(seed, TID_X + (micro << 32), shp)
    dy = normal(seed, TID_DY + (micro << 32), shp)
    if bf16:
        x, dy = round_to_bf16(x), round_to_bf16(dy)
    return x, dy
