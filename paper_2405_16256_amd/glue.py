"""PyTorch plumbing shared by the GPU parity tests, the smoke check and the benchmark:
moving seeded numpy inputs to the GPU, calling the C-ABI through the binding and
bringing results back as fp64.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2405_16256_amd import binding as hh
from paper_2405_16256_amd import inputs as I

DEV = "cuda:0"


def to_dev(a: np.ndarray, bf16: bool) -> torch.Tensor:
    if bf16:
        bits = torch.from_numpy(I.f32_to_bf16_bits(a).view(np.int16)).to(DEV)
        return bits.view(torch.bfloat16).reshape(a.shape)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    den = np.linalg.norm(ref.ravel())
    return float(np.linalg.norm((got - ref).ravel()) / (den if den > 0 else 1.0))


class DeviceLayer:
    """Device copies of one layer's parameters and fp32 gradient buffers.
    packed=True keeps wq|wk|wv and w_gate|w_up (and their gradients) in single allocations."""

    def __init__(self, w: dict, s: I.LayerShape, bf16: bool, packed: bool = True):
        self.s, self.bf16 = s, bf16
        dt = torch.bfloat16 if bf16 else torch.float32
        H, A, Akv, F = s.hidden, s.attn, s.attn_kv, s.ffn
        self.w, self.g = {}, {}
        if packed:
            wqkv = torch.empty(A + 2 * Akv, H, dtype=dt, device=DEV)
            wgu = torch.empty(2 * F, H, dtype=dt, device=DEV)
            gqkv = torch.zeros(A + 2 * Akv, H, dtype=torch.float32, device=DEV)
            ggu = torch.zeros(2 * F, H, dtype=torch.float32, device=DEV)
            for n, (lo, hi) in (("wq", (0, A)), ("wk", (A, A + Akv)), ("wv", (A + Akv, A + 2 * Akv))):
                self.w[n] = wqkv[lo:hi]
                self.g[n] = gqkv[lo:hi]
            for i, n in enumerate(("w_gate", "w_up")):
                self.w[n] = wgu[i * F:(i + 1) * F]
                self.g[n] = ggu[i * F:(i + 1) * F]
            self._keep = (wqkv, wgu, gqkv, ggu)
        for n in hh.WEIGHT_FIELDS:
            src = to_dev(w[n], bf16)
            if n in self.w:
                self.w[n].copy_(src)
            else:
                self.w[n] = src
                self.g[n] = torch.zeros(w[n].shape, dtype=torch.float32, device=DEV)
        self.wstruct = hh.make_weights(self.w)
        self.gstruct = hh.make_grads(self.g)

    def grads_np(self) -> dict:
        return {n: to_np(self.g[n]) for n in hh.WEIGHT_FIELDS}


def cfg_of(s: I.LayerShape, bf16: bool) -> hh.hh_layer_cfg:
    return hh.make_cfg(s.hidden, s.n_heads, s.head_dim, s.ffn, s.seq, s.micro_batch, s.rms_eps, s.rope_base,
                       hh.HH_BF16 if bf16 else hh.HH_F32, n_kv_heads=s.kv_heads)


def stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def run_layer(ctx, s: I.LayerShape, bf16: bool, layer: DeviceLayer, x_np, dy_np, accumulate=False):
    """One hh_layer_fwd + hh_layer_bwd through the C-ABI.  -> (y, dx) as fp64 numpy, saved buffer."""
    cfg = cfg_of(s, bf16)
    saved_b, ws_b = hh.hh_layer_sizes(cfg)
    dt = torch.bfloat16 if bf16 else torch.float32
    x, dy = to_dev(x_np, bf16), to_dev(dy_np, bf16)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    saved = torch.empty(saved_b, dtype=torch.uint8, device=DEV)
    ws = torch.empty(ws_b, dtype=torch.uint8, device=DEV)
    st = stream_ptr()
    hh.hh_layer_fwd(ctx, cfg, layer.wstruct, x, y, saved, ws, st)
    hh.hh_layer_bwd(ctx, cfg, layer.wstruct, x, saved, dy, dx, layer.gstruct, accumulate, ws, st)
    torch.cuda.synchronize()
    assert y.dtype == dt
    return to_np(y), to_np(dx), saved
