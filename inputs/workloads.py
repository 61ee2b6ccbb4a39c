"""Seeded synthetic inputs for the intermediate-layer token-recall path.

This module only *draws data*: query states, a key cache with planted needle
spans, and the workload parameters (pooling kernel sizes, budget).  It holds
none of the method's arithmetic (no logits, no softmax, no pooling, no
selection) so that the CPU oracle and the GPU path can both be fed from it
without sharing any of their own code.

The workloads stand in for the long-context retrieval suites the paper
evaluates on (its RULER / needle runs, Section 4 and the needle appendix):
shapes are Llama-3.1-8B's (32 query heads, 8 kv heads, head_dim 128), context
lengths 4K..1M, budget 4K; values are synthetic.

Recipe (all draws from numpy's default_rng, PCG64):
  data seed  = 1000 + cfg      (directions, channel scales, Q, K, needle noise)
  span seed  = 2000 + cfg      (span lengths and offsets)
  c_g   ~ N(0,1)^d                      one common query direction per kv group
  sig_g ~ U(0.5,2)^d  (cfg >= 3) or 1   per-channel scale of a kv group
  Q[h,i,:]  = (sqrt(1-rho^2) * N(0,1) + rho * c_g) * sig_g,   rho = 0.5
  K[g,t,:]  = N(0,1) * sig_g                                   (background)
  mhat_g    = mean of Q over the G heads and Lq tokens of group g, rescaled to
              the RMS of a background key of that group
  K[g,t,:]  = 0.8 * mhat_g + 0.2 * sig_g * N(0,1)              (t in a span)
Spans do not overlap; every kv head carries the needle at the same positions.
For the bf16 workloads Q and K are rounded to bf16 (round to nearest even) and
the *rounded* bit patterns are what both consumers receive.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

RHO = 0.5
NEEDLE_MIX = (0.8, 0.2)


@dataclass(frozen=True)
class Workload:
    name: str
    cfg: int
    L: int
    Lq: int
    Hq: int
    Hkv: int
    d: int
    dtype: str                      # "f32" or "bf16"
    pool_kernels: Tuple[int, ...]
    budget: int
    n_spans: int
    span_len: Tuple[int, int]       # inclusive range of span lengths
    channel_scale: bool


CONFIGS = {
    1: Workload("cfg1_tiny_4k", 1, 4096, 32, 32, 8, 128, "f32", (3, 7, 15), 256, 2, (32, 32), False),
    2: Workload("cfg2_32k", 2, 32768, 64, 32, 8, 128, "bf16", (3, 7, 15, 31), 4096, 4, (64, 64), False),
    3: Workload("cfg3_128k", 3, 131072, 128, 32, 8, 128, "bf16", (3, 7, 15, 31), 4096, 16, (64, 64), True),
    4: Workload("cfg4_512k", 4, 524288, 128, 32, 8, 128, "bf16", (3, 7, 15, 31), 4096, 32, (64, 256), True),
    5: Workload("cfg5_1m", 5, 1048576, 256, 32, 8, 128, "bf16", (1, 3, 7, 15, 31), 4096, 64, (64, 256), True),
}


@dataclass
class Inputs:
    workload: Workload
    q: np.ndarray                   # [Hq, Lq, d]  float32, or uint16 bf16 bit patterns
    k: np.ndarray                   # [Hkv, L, d]  same element type as q
    spans: List[Tuple[int, int]] = field(default_factory=list)   # (start, length)

    @property
    def needle_mask(self) -> np.ndarray:
        m = np.zeros(self.workload.L, dtype=bool)
        for s, n in self.spans:
            m[s:s + n] = True
        return m


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 exactly."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_float(a: np.ndarray) -> np.ndarray:
    """Exact float32 view of a generated array whatever its storage type."""
    return bf16_bits_to_f32(a) if a.dtype == np.uint16 else a


def place_spans(rng: np.random.Generator, L: int, n_spans: int, lo: int, hi: int) -> List[Tuple[int, int]]:
    """Non-overlapping spans with lengths in [lo, hi] and uniform random offsets."""
    spans: List[Tuple[int, int]] = []
    taken = np.zeros(L, dtype=bool)
    lens = rng.integers(lo, hi + 1, size=n_spans)
    for n in lens:
        n = int(min(n, L))
        for _ in range(10000):
            s = int(rng.integers(0, L - n + 1))
            if not taken[s:s + n].any():
                taken[s:s + n] = True
                spans.append((s, n))
                break
        else:
            raise RuntimeError("could not place span; context too crowded")
    spans.sort()
    return spans


def generate(wl: Workload, data_seed: int | None = None, span_seed: int | None = None,
             spans: List[Tuple[int, int]] | None = None) -> Inputs:
    """Draw Q, K and needle spans for a workload (see module docstring for the recipe)."""
    rng = np.random.default_rng(1000 + wl.cfg if data_seed is None else data_seed)
    rng_span = np.random.default_rng(2000 + wl.cfg if span_seed is None else span_seed)
    G = wl.Hq // wl.Hkv
    d = wl.d
    if spans is None:
        spans = place_spans(rng_span, wl.L, wl.n_spans, *wl.span_len) if wl.n_spans else []

    c = rng.standard_normal((wl.Hkv, d), dtype=np.float32)
    if wl.channel_scale:
        sig = rng.uniform(0.5, 2.0, size=(wl.Hkv, d)).astype(np.float32)
    else:
        sig = np.ones((wl.Hkv, d), dtype=np.float32)

    q = rng.standard_normal((wl.Hq, wl.Lq, d), dtype=np.float32)
    q *= np.float32(np.sqrt(1.0 - RHO * RHO))
    for g in range(wl.Hkv):
        q[g * G:(g + 1) * G] += np.float32(RHO) * c[g]
        q[g * G:(g + 1) * G] *= sig[g]

    to_store = f32_to_bf16_bits if wl.dtype == "bf16" else (lambda a: np.ascontiguousarray(a, dtype=np.float32))
    k_out = np.empty((wl.Hkv, wl.L, d), dtype=np.uint16 if wl.dtype == "bf16" else np.float32)
    for g in range(wl.Hkv):
        kg = rng.standard_normal((wl.L, d), dtype=np.float32)
        kg *= sig[g]
        mean_q = q[g * G:(g + 1) * G].reshape(-1, d).mean(axis=0)
        rms_bg = np.sqrt(np.mean(sig[g].astype(np.float64) ** 2))
        rms_m = np.sqrt(np.mean(mean_q.astype(np.float64) ** 2))
        mhat = (mean_q * np.float32(rms_bg / max(rms_m, 1e-30))).astype(np.float32)
        for s, n in spans:
            noise = rng.standard_normal((n, d), dtype=np.float32) * sig[g]
            kg[s:s + n] = np.float32(NEEDLE_MIX[0]) * mhat + np.float32(NEEDLE_MIX[1]) * noise
        k_out[g] = to_store(kg)
        del kg
    return Inputs(wl, to_store(q), k_out, list(spans))


def custom(L: int, Lq: int, Hq: int, Hkv: int, d: int, dtype: str = "bf16",
           pool_kernels: Tuple[int, ...] = (3, 7, 15), budget: int = 64, n_spans: int = 0,
           span_len: Tuple[int, int] = (8, 8), channel_scale: bool = False,
           seed: int = 0, name: str = "custom") -> Inputs:
    """Same recipe at an arbitrary shape; `seed` replaces the cfg number in both seeds."""
    wl = Workload(name, 0, L, Lq, Hq, Hkv, d, dtype, tuple(pool_kernels), budget,
                  n_spans, span_len, channel_scale)
    return generate(wl, data_seed=1000 + seed, span_seed=2000 + seed)


def config(cfg: int) -> Inputs:
    return generate(CONFIGS[cfg])
