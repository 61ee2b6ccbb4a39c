"""CPU oracle for the DCA re-RoPE of the retrieval layer's key cache (numpy, fp64, plain definitions).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
cpu_baseline leg.  The product path never calls it.

Follows the second DCA equation of the paper (Section 3.3, "Dual Chunk Attention"): before the
recall step the keys of prefill chunk i are rotated by R(D_i), D_i being the distance between
chunk i and chunk N_C - 1, for i < N_C - 1 only; chunk N_C - 1 is the positional base because the
last chunk may be shorter.

Readings taken where the paper is silent:
  * chunks are numbered 1..N_C in prefill order; chunk 1 holds `first_extra` more tokens than the
    chunk size (the sink part, "the first chunk with additional S" of the default settings), the
    last chunk may be shorter; N_C = max(1, ceil((L - first_extra) / chunk));
  * D_i = (N_C - 1 - i) * chunk tokens for i = 1 .. N_C - 2; chunks N_C - 1 and N_C are unchanged;
  * R(D) is the rotary position embedding's rotation by D positions: pair j of a key vector is
    turned by the angle D * inv_freq[j], (x, y) -> (x cos - y sin, y cos + x sin), which moves a key
    embedded at position p to position p + D;
  * inv_freq[j] = base^(-2j/d) unless the caller passes its own table (models with scaled
    frequencies); pair j is (x[j], x[j + d/2]) in the half-split layout of the Llama family
    (PAIR_HALF, default) or (x[2j], x[2j+1]) in the interleaved layout (PAIR_INTERLEAVED);
  * the result is returned unrounded (fp64); a bf16 cache is compared after rounding.
"""
from __future__ import annotations

from typing import List, Optional, Tuple

import numpy as np

PAIR_HALF, PAIR_INTERLEAVED = 0, 1


def default_inv_freq(d: int, base: float = 10000.0) -> np.ndarray:
    """inv_freq[j] = base^(-2j/d), j = 0 .. d/2 - 1 (fp64)."""
    if d < 2 or d % 2:
        raise ValueError("head dimension must be even")
    return np.float64(base) ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)


def chunk_bounds(L: int, chunk: int, first_extra: int = 0) -> List[Tuple[int, int]]:
    """Token ranges [start, end) of the prefill chunks, in order."""
    if L < 1 or chunk < 1 or first_extra < 0:
        raise ValueError("L and chunk must be positive, first_extra non-negative")
    n = max(1, -(-(L - first_extra) // chunk))
    out = []
    for c in range(n):
        start = 0 if c == 0 else first_extra + c * chunk
        end = min(L, first_extra + (c + 1) * chunk)
        out.append((start, end))
    return out


def chunk_distances(n_chunks: int, chunk: int) -> List[int]:
    """D_i in tokens for the chunks in order (0 for the last two)."""
    return [max(0, n_chunks - 2 - c) * chunk for c in range(n_chunks)]


def rotate(x: np.ndarray, distance: float, inv_freq: np.ndarray, pairing: int = PAIR_HALF) -> np.ndarray:
    """R(distance) applied to the last axis of x (fp64 in, fp64 out)."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    ang = np.float64(distance) * np.asarray(inv_freq, dtype=np.float64)
    if ang.shape != (d // 2,):
        raise ValueError("inv_freq must have d/2 entries")
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    if pairing == PAIR_HALF:
        a, b = x[..., :d // 2], x[..., d // 2:]
        out[..., :d // 2] = a * c - b * s
        out[..., d // 2:] = b * c + a * s
    elif pairing == PAIR_INTERLEAVED:
        a, b = x[..., 0::2], x[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = b * c + a * s
    else:
        raise ValueError("unknown pairing")
    return out


def _widen(k: np.ndarray) -> np.ndarray:
    if k.dtype == np.uint16:  # bf16 bit patterns
        return (k.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return k.astype(np.float64)


def rerope_keys(k: np.ndarray, chunk: int, first_extra: int = 0, base: float = 10000.0,
                inv_freq: Optional[np.ndarray] = None, pairing: int = PAIR_HALF) -> np.ndarray:
    """The re-RoPE'd key cache, fp64 [Hkv, L, d]; k is float32 or uint16 bf16 bit patterns."""
    if k.ndim != 3:
        raise ValueError("k is [Hkv, L, d]")
    _, L, d = k.shape
    freq = default_inv_freq(d, base) if inv_freq is None else np.asarray(inv_freq, dtype=np.float64)
    x = _widen(k)
    bounds = chunk_bounds(L, chunk, first_extra)
    out = x.copy()
    for (start, end), dist in zip(bounds, chunk_distances(len(bounds), chunk)):
        if dist:
            out[:, start:end, :] = rotate(x[:, start:end, :], dist, freq, pairing)
    return out
