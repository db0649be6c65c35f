"""Seeded synthetic inputs generated directly in device memory, for the configurations whose weights and KV cache
are too large to draw on the host (7B / 14B shapes).  Inputs only: no arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from .gen import ModelShape, rope_table


def make_weights_device(shape: ModelShape, seed: int, n_layers: int | None = None, std: float = 0.02,
                        device: str = "cuda:0") -> dict:
    """Random-init decoder weights N(0, std) rounded to bf16, as torch tensors on the device.
    Same dictionary layout as hs_inputs.make_weights (matrices [out_features, in_features])."""
    L = shape.n_layers if n_layers is None else n_layers
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    d, F, V = shape.d_model, shape.d_ffn, shape.vocab
    qh = shape.n_q_heads * shape.head_dim

    def mat(rows, cols):
        out = torch.empty(rows, cols, dtype=torch.bfloat16, device=device)
        step = max(1, (1 << 27) // cols)
        for r in range(0, rows, step):
            e = min(rows, r + step)
            out[r:e] = (torch.randn(e - r, cols, generator=g, device=device, dtype=torch.float32) * std).to(torch.bfloat16)
        return out

    ones = lambda: torch.ones(d, dtype=torch.float32, device=device)
    w = {"embed": mat(V, d), "lm_head": mat(V, d), "norm_f": ones(),
         "wqkv": [], "wo": [], "wgate": [], "wup": [], "wdown": [], "norm1": [], "norm2": []}
    for _ in range(L):
        w["wqkv"].append(mat(shape.qkv_rows, d))
        w["wo"].append(mat(d, qh))
        w["wgate"].append(mat(F, d))
        w["wup"].append(mat(F, d))
        w["wdown"].append(mat(d, F))
        w["norm1"].append(ones())
        w["norm2"].append(ones())
    return w


def weights_to_host(w: dict) -> dict:
    """Bit-exact host copy (uint16 bf16 bits / float32) of device weights, for the oracle."""
    def conv(t):
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()
    return {k: ([conv(x) for x in v] if isinstance(v, list) else conv(v)) for k, v in w.items()}


def fill_kv_random(kc: torch.Tensor, vc: torch.Tensor, seed: int, std: float, chunk: int = 1 << 28):
    """Fill a paged KV cache (int16 storage of bf16 bits) with N(0, std) values: a stand-in for the K/V a prefill of
    random context tokens would have written (same size, dtype and value scale)."""
    g = torch.Generator(device=kc.device)
    g.manual_seed(seed)
    for t in (kc, vc):
        flat = t.view(-1).view(torch.bfloat16)
        for s in range(0, flat.numel(), chunk):
            e = min(flat.numel(), s + chunk)
            flat[s:e] = (torch.randn(e - s, generator=g, device=kc.device, dtype=torch.float32) * std).to(torch.bfloat16)


def rope_device(max_pos: int, head_dim: int, device: str = "cuda:0") -> torch.Tensor:
    return torch.from_numpy(rope_table(max_pos, head_dim)).to(device)
