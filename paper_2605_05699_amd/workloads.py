"""Seeded synthetic KV-cache workloads (inputs only).

This module holds no part of the method: no transform, no quantizer, no sign
generator.  It only describes the five cache shapes the library is measured
on and draws their inputs, so that the HIP path, the tests and the CPU oracle
are all handed the same arrays.

The paper evaluates on activations of SmolLM2 / Qwen2.5-1.5B / Gemma-3 1B over
Cosmopedia text (Sec. 4.1); neither weights nor text are used here.  The
tensors below take the shapes of those caches (layers x KV heads x head_dim,
prefix lengths) and the structure the paper reports for them: a near-Gaussian
bulk, a few persistent outlier channels in K (Sec. 5.6), heavy-tailed
per-channel scales.

A "plan" is one (layer, K|V) pair: plan index = 2 * layer + kind, kind 0 = K,
1 = V.  Every plan has its own sign seed and its own lambda vector.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class KVWorkload:
    name: str
    index: int               # 1-based position in the list of configurations
    d: int                   # head_dim
    g: int                   # quantization group size
    layers: int
    kv_heads: int
    batch: int
    tokens: int              # tokens per sequence held in the cache
    outlier_frac: float      # fraction of channels that are outliers (at least 1 if > 0)
    outlier_count: int       # explicit count (overrides outlier_frac when > 0)
    outlier_gain: float
    outliers_k_only: bool
    channel_lognormal_sigma: float   # > 0: per-channel scale ~ lognormal(0, sigma)
    append_tokens: int = 0   # decode-step append: new tokens per sequence per step

    @property
    def n_plans(self) -> int:
        return 2 * self.layers

    @property
    def vectors_per_plan(self) -> int:
        return self.batch * self.kv_heads * self.tokens

    @property
    def append_vectors_per_plan(self) -> int:
        return self.batch * self.kv_heads * self.append_tokens

    @property
    def total_vectors(self) -> int:
        return self.n_plans * self.vectors_per_plan

    @property
    def base_seed(self) -> int:
        return 1000 + self.index

    def plan_seed(self, plan: int) -> int:
        return self.base_seed * 1_000_003 + plan


WORKLOADS = {
    w.name: w for w in [
        KVWorkload("tiny", 1, d=128, g=32, layers=1, kv_heads=1, batch=1, tokens=256,
                   outlier_frac=0.0, outlier_count=4, outlier_gain=20.0, outliers_k_only=False,
                   channel_lognormal_sigma=0.0),
        KVWorkload("qwen2.5-1.5b-4k", 2, d=128, g=32, layers=28, kv_heads=2, batch=1, tokens=4096,
                   outlier_frac=0.01, outlier_count=0, outlier_gain=30.0, outliers_k_only=True,
                   channel_lognormal_sigma=0.0),
        KVWorkload("gemma3-1b-4k", 3, d=256, g=32, layers=26, kv_heads=1, batch=1, tokens=4096,
                   outlier_frac=0.0, outlier_count=0, outlier_gain=1.0, outliers_k_only=False,
                   channel_lognormal_sigma=1.0),
        KVWorkload("decode-d96", 4, d=96, g=32, layers=32, kv_heads=8, batch=64, tokens=8192,
                   outlier_frac=0.0, outlier_count=1, outlier_gain=20.0, outliers_k_only=False,
                   channel_lognormal_sigma=0.0, append_tokens=1),
        KVWorkload("llama3-70b-128k", 5, d=128, g=32, layers=80, kv_heads=8, batch=1, tokens=131072,
                   outlier_frac=0.01, outlier_count=0, outlier_gain=30.0, outliers_k_only=True,
                   channel_lognormal_sigma=0.0),
    ]
}


def plan_constants(w: KVWorkload, plan: int):
    """(sign_seed, lambda float32[d], channel_gain float32[d]) of one plan, from its seed."""
    rng = np.random.RandomState(w.plan_seed(plan) % (2 ** 32))
    lam = np.exp(0.5 * rng.standard_normal(w.d)).astype(np.float32)   # lognormal(0, 0.5)
    gain = np.ones(w.d, dtype=np.float32)
    is_k = (plan % 2 == 0)
    n_out = w.outlier_count if w.outlier_count > 0 else (
        max(1, int(round(w.outlier_frac * w.d))) if w.outlier_frac > 0 else 0)
    if n_out and (is_k or not w.outliers_k_only):
        idx = rng.choice(w.d, size=n_out, replace=False)
        gain[idx] *= w.outlier_gain
    if w.channel_lognormal_sigma > 0:
        gain *= np.exp(w.channel_lognormal_sigma * rng.standard_normal(w.d)).astype(np.float32)
    sign_seed = w.plan_seed(plan)
    return sign_seed, lam, gain


def fill_kv(out: torch.Tensor, w: KVWorkload, plan: int, chunk: int = 1 << 20) -> torch.Tensor:
    """Fill ``out`` ([n, d] fp16, any device) with plan ``plan``'s values: N(0,1) * channel gain."""
    assert out.dtype == torch.float16 and out.dim() == 2 and out.shape[1] == w.d
    _, _, gain = plan_constants(w, plan)
    gen = torch.Generator(device=out.device)
    gen.manual_seed(w.plan_seed(plan))
    gain_t = torch.from_numpy(gain).to(out.device)
    n = out.shape[0]
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        v = torch.randn(hi - lo, w.d, generator=gen, device=out.device, dtype=torch.float32)
        out[lo:hi] = (v * gain_t).to(torch.float16)
    return out


def make_kv(w: KVWorkload, plan: int, n_vec: int | None = None, device="cpu") -> torch.Tensor:
    """A fresh [n_vec, d] fp16 tensor of plan ``plan`` (default: the plan's full size)."""
    n = w.vectors_per_plan if n_vec is None else n_vec
    return fill_kv(torch.empty(n, w.d, dtype=torch.float16, device=device), w, plan)


def gaussian_with_outliers(n: int, d: int, seed: int, outliers: int = 1, gain: float = 20.0) -> np.ndarray:
    """Small CPU helper for tests at arbitrary d: [n, d] fp16, N(0,1) with ``outliers`` channels x gain."""
    rng = np.random.RandomState(seed)
    x = rng.standard_normal((n, d))
    if outliers:
        x[:, rng.choice(d, size=outliers, replace=False)] *= gain
    return x.astype(np.float16)


def lognormal_lambda(d: int, seed: int, sigma: float = 0.5) -> np.ndarray:
    return np.exp(sigma * np.random.RandomState(seed).standard_normal(d)).astype(np.float32)
