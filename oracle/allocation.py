"""CPU oracle for the context-allocation part of the recall path (numpy, plain definitions).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
cpu_baseline leg.  The product path never calls it.

Follows Algorithm 1 ("Context Allocation") of the paper, Section 3.2, in the form the
target workloads use: one stride-1 max-pooling per kernel size instead of the printed
strided-max then average pooling, so a pooled index is the token index itself.

Readings taken where the algorithm is silent:
  * pooling windows are clipped to [0, L) ("same" padding; padding never wins a max);
  * the per-kernel budget B_c = B / n is made integral by floor, the first (B mod n)
    kernels taking one more, so exactly B indices come out;
  * kernels are processed in the order given (order matters through the allocated set I);
  * candidates are ranked by (pooled score descending, token index ascending);
  * all not-yet-allocated tokens are candidates (no top-K_m cap), so a kernel always
    finds its share while unallocated tokens remain;
  * no sink part: I starts empty.
Decisions are taken in the precision of the array passed in (pass float32 to decide as the
GPU path does).
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np


def max_pool_same(score: np.ndarray, w: int) -> np.ndarray:
    """pooled[t] = max(score[u] : |u - t| <= (w-1)/2, 0 <= u < L); the MaxPooling step of
    Algorithm 1 at stride 1."""
    if w < 1 or w % 2 == 0:
        raise ValueError("kernel size must be odd and >= 1")
    L = score.shape[0]
    r = (w - 1) // 2
    pooled = score.copy()
    for s in range(1, r + 1):
        if s >= L:
            break
        # neighbour s to the right and s to the left, where they exist
        pooled[:L - s] = np.maximum(pooled[:L - s], score[s:])
        pooled[s:] = np.maximum(pooled[s:], score[:L - s])
    return pooled


def split_budget(budget: int, n: int) -> List[int]:
    """B_c of Algorithm 1 made integral: floor(B/n), the first B mod n kernels get one more."""
    if budget < 1 or n < 1:
        raise ValueError("budget and kernel count must be positive")
    base, rem = divmod(budget, n)
    return [base + (1 if j < rem else 0) for j in range(n)]


def allocate(score: np.ndarray, pool_kernels: Sequence[int], budget: int) -> np.ndarray:
    """Algorithm 1: per kernel size pool, rank, add the first B_j tokens not yet in I;
    return I sorted ascending (int64)."""
    L = score.shape[0]
    shares = split_budget(budget, len(pool_kernels))
    allocated = np.zeros(L, dtype=bool)
    token = np.arange(L)
    for w, share in zip(pool_kernels, shares):
        pooled = max_pool_same(score, int(w))
        # rank every token by (pooled descending, index ascending)
        order = np.lexsort((token, -pooled.astype(np.float64)))
        free = order[~allocated[order]]
        take = free[:share]
        allocated[take] = True
    return np.flatnonzero(allocated).astype(np.int64)


def thresholds(score: np.ndarray, pool_kernels: Sequence[int], budget: int):
    """For the index-set comparison rule: replay Algorithm 1 and report, per kernel, the pooled
    vector and the pooled value of the last token that kernel admitted (its threshold), or None
    when the kernel admitted nothing."""
    L = score.shape[0]
    shares = split_budget(budget, len(pool_kernels))
    allocated = np.zeros(L, dtype=bool)
    token = np.arange(L)
    out = []
    for w, share in zip(pool_kernels, shares):
        pooled = max_pool_same(score, int(w))
        order = np.lexsort((token, -pooled.astype(np.float64)))
        free = order[~allocated[order]]
        take = free[:share]
        allocated[take] = True
        out.append((pooled, float(pooled[take[-1]]) if take.size else None))
    return out
