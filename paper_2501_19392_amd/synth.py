"""Seeded synthetic inputs shaped like the paper's Llama-3.x KV workloads.

This module only *produces inputs* (KV tensors, sign vectors, a grid, predictor
weights).  It holds none of the encode/decode arithmetic; the HIP library and
the CPU oracle are both fed from here and neither depends on the other.

The paper (Sect. 4) evaluates on Llama-3.x / Qwen-2.5 KV caches computed from
RedPajama, WikiText-2 and LongBench text; none of that is available offline, so
these generators stand in for it.  What is kept from the paper: the tensor
shapes (8 KV heads x 128, 28/32/80 layers, 8192 .. 2^17 tokens), a few outlier
channels (Sect. 2 on KV statistics), and a strong, roughly linear dependence
between consecutive layers (Sect. 3.1: linear probes explain one half to nine
tenths of the variance).

Recipe.  Layer 0: x = n * a with n ~ N(0,1) i.i.d., a a per-channel log-normal
(sigma = 1) scale multiplied by 10 on two seeded outlier channels.  Layer l+1:
x = 0.7 * (layer l) @ W_true + 0.3 * fresh noise of the same recipe, W_true a
seeded random orthogonal matrix.  Keys and values use separate streams.
Seeds: BASE_SEED + 7*layer + {K:0, V:1, W_k:2, signs:3, grid:4, W_v:5}.
"""
from __future__ import annotations

from dataclasses import dataclass
from functools import lru_cache

import numpy as np
import torch

BASE_SEED = 20250131
_K, _V, _WK, _SIGNS, _GRID, _WV = 0, 1, 2, 3, 4, 5


def _seed(layer: int, what: int) -> int:
    return BASE_SEED + 7 * layer + what


@dataclass(frozen=True)
class Config:
    name: str
    layers: int
    kv_heads: int
    head_dim: int
    tokens: int
    dtype: str            # "bf16" | "fp32"
    n_codewords: int = 16
    corr: float = 0.7

    @property
    def d(self) -> int:
        return self.kv_heads * self.head_dim


TINY = Config("tiny", layers=2, kv_heads=2, head_dim=128, tokens=256, dtype="fp32")
LLAMA32_3B = Config("llama3.2-3b-kv", layers=28, kv_heads=8, head_dim=128, tokens=8192, dtype="bf16")
LLAMA31_8B = Config("llama3.1-8b-kv", layers=32, kv_heads=8, head_dim=128, tokens=32768, dtype="bf16")
LLAMA31_70B = Config("llama3.1-70b-kv", layers=80, kv_heads=8, head_dim=128, tokens=131072, dtype="bf16")


def torch_dtype(dtype: str) -> torch.dtype:
    return {"bf16": torch.bfloat16, "fp32": torch.float32}[dtype]


# ---------------------------------------------------------------- small pieces
def rht_signs(kv_heads: int, head_dim: int, layer: int, which: str) -> np.ndarray:
    """+-1 per channel, int8 [kv_heads, head_dim]; separate for keys and values."""
    rng = np.random.Generator(np.random.PCG64(_seed(layer, _SIGNS) * 2 + (0 if which == "k" else 1)))
    return (rng.integers(0, 2, size=(kv_heads, head_dim)) * 2 - 1).astype(np.int8)


def lloyd_codebook(n: int, p: int = 2, iters: int = 50, log2_samples: int = 16, seed: int | None = None) -> np.ndarray:
    """Cached front of _lloyd_codebook (the grid depends only on its arguments)."""
    return _lloyd_codebook(n, p, iters, log2_samples, seed).copy()


@lru_cache(maxsize=None)
def _lloyd_codebook(n: int, p: int, iters: int, log2_samples: int, seed: int | None) -> np.ndarray:
    """A grid of n points in R^p for N(0, I_p) inputs: plain Lloyd iterations.

    Initial centres are the first n samples; an empty cell keeps its centre; the
    result is sorted lexicographically so that indices are canonical.  fp32 out.
    """
    rng = np.random.Generator(np.random.PCG64(_seed(0, _GRID) if seed is None else seed))
    x = rng.standard_normal((1 << log2_samples, p))
    c = x[:n].copy()
    for _ in range(iters):
        d = ((x[:, None, :] - c[None, :, :]) ** 2).sum(-1)
        a = d.argmin(1)
        for j in range(n):
            m = a == j
            if m.any():
                c[j] = x[m].mean(0)
    order = np.lexsort(tuple(c[:, k] for k in reversed(range(p))))
    return c[order].astype(np.float32)


def channel_scales(d: int, layer: int, which: int, device="cpu") -> torch.Tensor:
    rng = np.random.Generator(np.random.PCG64(_seed(layer, which) + 1000003))
    a = np.exp(rng.standard_normal(d))
    out = rng.choice(d, size=2, replace=False)
    a[out] *= 10.0
    return torch.from_numpy(a).to(device)


def random_orthogonal(d: int, seed: int, device="cpu", dtype=torch.float64) -> torch.Tensor:
    g = torch.Generator(device="cpu").manual_seed(seed)
    a = torch.randn(d, d, generator=g, dtype=torch.float64)
    q, r = torch.linalg.qr(a)
    q = q * torch.sign(torch.diagonal(r))[None, :]
    return q.to(device=device, dtype=dtype)


# ---------------------------------------------------------------- KV streams
class KVStream:
    """Generates (K_l, V_l) layer by layer on `device`, never holding more than
    two layers.  Values are rounded to the config's storage dtype.  `work` is
    the dtype the recurrence runs in (fp64 for the tiny config, fp32 on a GPU)."""

    def __init__(self, cfg: Config, device="cpu", work=torch.float64, tokens: int | None = None):
        self.cfg, self.device, self.work = cfg, torch.device(device), work
        self.tokens = cfg.tokens if tokens is None else tokens
        self.layer = -1
        self._k = self._v = None

    def _noise(self, layer: int, which: int) -> torch.Tensor:
        g = torch.Generator(device=self.device).manual_seed(_seed(layer, which))
        n = torch.randn(self.tokens, self.cfg.d, generator=g, device=self.device, dtype=self.work)
        return n * channel_scales(self.cfg.d, layer, which, self.device).to(self.work)[None, :]

    def w_true(self, layer: int, which: str) -> torch.Tensor:
        """Orthogonal map taking layer-1's tensor to this layer's (layer >= 1)."""
        return random_orthogonal(self.cfg.d, _seed(layer, _WK if which == "k" else _WV), self.device, self.work)

    def next(self):
        self.layer += 1
        l, c = self.layer, self.cfg.corr
        if l == 0:
            k, v = self._noise(0, _K), self._noise(0, _V)
        else:
            k = c * (self._k @ self.w_true(l, "k")) + (1 - c) * self._noise(l, _K)
            v = c * (self._v @ self.w_true(l, "v")) + (1 - c) * self._noise(l, _V)
        self._k, self._v = k, v
        sd = torch_dtype(self.cfg.dtype)
        shape = (self.tokens, self.cfg.kv_heads, self.cfg.head_dim)
        return k.to(sd).reshape(shape), v.to(sd).reshape(shape)


def analytic_predictors(stream: KVStream, layer: int):
    """Predictor weights that match the generator: w_k = c * W_true_k^T and
    w_v = [c * W_true_v^T | 0] plus a small seeded dense perturbation so that
    every block of the weights matters to the result.  Returned in fp32,
    [d_out, d_in] layout (w_v inputs: previous values first, then keys)."""
    cfg = stream.cfg
    d = cfg.d
    g = torch.Generator(device="cpu").manual_seed(_seed(layer, _WK) + 500009)
    wk = cfg.corr * stream.w_true(layer, "k").T.float().cpu()
    wv = torch.cat([cfg.corr * stream.w_true(layer, "v").T.float().cpu(), torch.zeros(d, d)], dim=1)
    wk = wk + 0.05 / d ** 0.5 * torch.randn(d, d, generator=g)
    wv = wv + 0.05 / d ** 0.5 * torch.randn(d, 2 * d, generator=g)
    return wk.contiguous(), wv.contiguous()


def random_queries(batch: int, q_heads: int, head_dim: int, seed: int, dtype: str = "bf16", device="cpu") -> torch.Tensor:
    g = torch.Generator(device="cpu").manual_seed(seed)
    q = torch.randn(batch, q_heads, head_dim, generator=g, dtype=torch.float32)
    return q.to(torch_dtype(dtype)).to(device)
