"""Seeded generators for every synthetic input of the five benchmark configurations.

All arrays are plain numpy.  Weights are drawn once here (N(0, 0.02), rounded to
bf16 round-to-nearest-even, returned as uint16 bit patterns) and handed to both
the oracle and the HIP path, so the two never re-draw them independently.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    """Dense pre-norm decoder shape (RMSNorm, RoPE, GQA, SwiGLU, untied LM head)."""

    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def dense_params(self) -> int:
        per_layer = (self.d_model * self.qkv_rows + self.n_q_heads * self.head_dim * self.d_model
                     + 3 * self.d_model * self.d_ffn)
        return self.n_layers * per_layer + self.d_model * self.vocab

    @property
    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * 2 * self.n_layers


# The five model shapes of the benchmark configurations (1-indexed).
CONFIG_SHAPES = {
    1: ModelShape(2, 256, 4, 4, 64, 1024, 4096),
    2: ModelShape(28, 1536, 12, 2, 128, 8960, 151936),
    3: ModelShape(28, 3584, 28, 4, 128, 18944, 152064),
    4: ModelShape(28, 3584, 28, 4, 128, 18944, 152064),
    5: ModelShape(48, 5120, 40, 8, 128, 13824, 152064),
}


def config_seed(config: int) -> int:
    """One documented 64-bit seed per configuration."""
    return 0xC0FFEE00 + int(config)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32 (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for s in range(0, n, step):
        e = min(n, s + step)
        out[s:e] = bf16_bits(rng.standard_normal(e - s, dtype=np.float32) * np.float32(std))
    return out.reshape(shape)


def make_weights(shape: ModelShape, seed: int, n_layers: int | None = None,
                 norm_jitter: float = 0.0, std: float = 0.02) -> dict:
    """Random-init decoder weights.

    Every matrix is row-major [out_features, in_features], bf16 bits (uint16).
    `wqkv` stacks the q, k and v projections in that order.  Norm weights are
    float32; they are 1 unless `norm_jitter` > 0 (used by tests so that a
    dropped norm weight shows up).
    """
    L = shape.n_layers if n_layers is None else n_layers
    rng = np.random.default_rng(seed)
    d, F, V = shape.d_model, shape.d_ffn, shape.vocab
    qh = shape.n_q_heads * shape.head_dim

    def norm_w():
        w = np.ones(d, dtype=np.float32)
        if norm_jitter > 0:
            w += (rng.standard_normal(d, dtype=np.float32) * np.float32(norm_jitter))
        return w

    w = {
        "embed": _normal_bf16(rng, (V, d), std),
        "lm_head": _normal_bf16(rng, (V, d), std),
        "norm_f": norm_w(),
        "wqkv": [], "wo": [], "wgate": [], "wup": [], "wdown": [], "norm1": [], "norm2": [],
    }
    for _ in range(L):
        w["wqkv"].append(_normal_bf16(rng, (shape.qkv_rows, d), std))
        w["wo"].append(_normal_bf16(rng, (d, qh), std))
        w["wgate"].append(_normal_bf16(rng, (F, d), std))
        w["wup"].append(_normal_bf16(rng, (F, d), std))
        w["wdown"].append(_normal_bf16(rng, (d, F), std))
        w["norm1"].append(norm_w())
        w["norm2"].append(norm_w())
    return w


def rope_table(max_pos: int, head_dim: int, base: float = 10000.0) -> np.ndarray:
    """[max_pos, head_dim/2, 2] float32 (cos, sin), evaluated in float64 then rounded once."""
    half = head_dim // 2
    inv = base ** (-np.arange(half, dtype=np.float64) * 2.0 / head_dim)
    ang = np.arange(max_pos, dtype=np.float64)[:, None] * inv[None, :]
    return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)


def make_prompts(batch: int, length: int, vocab: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed ^ 0x5EED0001)
    return rng.integers(0, vocab, size=(batch, length), dtype=np.int64).astype(np.int32)


def mutate(r: np.ndarray, p_iid: float, p_span: float, vocab: int,
           rng: np.random.Generator) -> np.ndarray:
    """Previous-epoch version of rollout `r`.

    Walk `r` left to right.  With probability p_span/16.5 per position a span
    edit of length s ~ U{1..32} starts: a coin flip picks insertion (emit s
    uniform-random tokens) or deletion (skip s tokens of r).  Otherwise the
    token is copied, replaced by a uniform-random token with probability p_iid.
    (About p_span of the positions end up covered by span edits.)
    """
    out = []
    i, n = 0, len(r)
    p_start = p_span / 16.5
    while i < n:
        if p_start > 0 and rng.random() < p_start:
            s = int(rng.integers(1, 33))
            if rng.random() < 0.5:
                out.extend(rng.integers(0, vocab, size=s).tolist())
            else:
                i += s
            continue
        if rng.random() < p_iid:
            out.append(int(rng.integers(0, vocab)))
        else:
            out.append(int(r[i]))
        i += 1
    return np.asarray(out, dtype=np.int32)


def history_with_context(prompt: np.ndarray, response_hist: np.ndarray, window: int) -> np.ndarray:
    """History array as the draft step scans it: the last window-1 prompt tokens
    followed by the previous-epoch response, so that a match can be anchored on
    the end of the prompt before any response token exists."""
    ctx = np.asarray(prompt[-(window - 1):] if window > 1 else prompt[:0], dtype=np.int32)
    return np.concatenate([ctx, np.asarray(response_hist, dtype=np.int32)])


def lengths_uniform(batch: int, lo: int, hi: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed ^ 0x5EED0002)
    return rng.integers(lo, hi + 1, size=batch).astype(np.int32)


def lengths_lognormal(batch: int, median: float, sigma: float, lo: int, hi: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed ^ 0x5EED0003)
    x = np.exp(rng.normal(np.log(median), sigma, size=batch))
    return np.clip(np.rint(x), lo, hi).astype(np.int32)
