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
  * sink part (optional, as in the printed form): the first `sink` tokens are always allocated and take
    no part in the pooling (the scores handed to the pooling are score[sink:]); the budget B counts the
    other tokens.  sink = 0: I starts empty.
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


def allocate(score: np.ndarray, pool_kernels: Sequence[int], budget: int, sink: int = 0) -> np.ndarray:
    """Algorithm 1: I starts as the sink indices; per kernel size pool score[sink:], rank, add the first
    B_j tokens not yet in I; return I sorted ascending (int64)."""
    if sink < 0 or sink > score.shape[0]:
        raise ValueError("sink out of range")
    body = score[sink:]
    L = body.shape[0]
    shares = split_budget(budget, len(pool_kernels))
    allocated = np.zeros(L, dtype=bool)
    token = np.arange(L)
    for w, share in zip(pool_kernels, shares):
        pooled = max_pool_same(body, int(w))
        # rank every token by (pooled descending, index ascending)
        order = np.lexsort((token, -pooled.astype(np.float64)))
        free = order[~allocated[order]]
        take = free[:share]
        allocated[take] = True
    return np.concatenate([np.arange(sink), sink + np.flatnonzero(allocated)]).astype(np.int64)


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


# ---------------------------------------------------------------------------------------------
# Algorithm 1 as printed: strided max pooling, then stride-1 average pooling, one combination per
# (max kernel, average kernel) pair.
#
# Readings taken where the algorithm is silent:
#   * MaxPooling(size = stride = m) keeps floor(L/m) whole cells; the up to m-1 tokens after the last
#     whole cell are never candidates of that max kernel;
#   * AvgPooling(size = n, stride 1) returns one value per cell: the window of cell p is
#     [p - floor((n-1)/2), p + floor(n/2)], cells outside the array count as zero, and the sum is
#     divided by n.  The sum is taken in the array's own precision, left to right;
#   * "Select top K_m indices": K_m = floor(B/m) + 1 cells, ranked (value descending, cell ascending);
#   * "Map back": cell p stands for its m tokens p*m .. p*m+m-1, walked in ascending order;
#   * B_c = floor(B / (N_M*N_A)), the first B mod (N_M*N_A) combinations taking one more; a combination
#     stops early when its K_m cells are used up, so fewer than B tokens may come out;
#   * combinations run with the max kernel in the outer loop and the average kernel in the inner loop;
#   * sink part: the first `sink` tokens are always allocated and take no part in the pooling (the
#     scores handed to the pooling are score[sink:]); the budget B counts the other tokens.


def max_pool_strided(score: np.ndarray, m: int) -> np.ndarray:
    """cell[p] = max(score[p*m : p*m+m]) for the floor(L/m) whole cells (MaxPooling, size = stride = m)."""
    if m < 1:
        raise ValueError("max kernel must be >= 1")
    cells = score.shape[0] // m
    return score[:cells * m].reshape(cells, m).max(axis=1) if cells else score[:0].copy()


def avg_pool_same(x: np.ndarray, n: int) -> np.ndarray:
    """out[p] = (x[p-a] + ... + x[p+b]) / n with a = (n-1)//2, b = n//2, zeros outside, summed left to
    right in x's dtype (AvgPooling, size n, stride 1)."""
    if n < 1:
        raise ValueError("average kernel must be >= 1")
    Lc = x.shape[0]
    acc = np.zeros(Lc, dtype=x.dtype)
    for off in range(-((n - 1) // 2), n // 2 + 1):
        lo, hi = max(0, -off), min(Lc, Lc - off)       # cells p with 0 <= p + off < Lc
        if lo < hi:
            acc[lo:hi] = acc[lo:hi] + x[lo + off:hi + off]
    return acc / x.dtype.type(n)


def allocate_max_avg(score: np.ndarray, max_kernels: Sequence[int], avg_kernels: Sequence[int], budget: int,
                     sink: int = 0) -> np.ndarray:
    """Algorithm 1 with strided max pooling and average pooling; returns I sorted ascending (int64),
    the sink indices included."""
    L = score.shape[0]
    if sink < 0 or sink > L:
        raise ValueError("sink out of range")
    body = score[sink:]
    Lb = body.shape[0]
    shares = split_budget(budget, len(max_kernels) * len(avg_kernels))
    allocated = np.zeros(Lb, dtype=bool)
    combo = 0
    for m in max_kernels:
        m = int(m)
        cells = max_pool_strided(body, m)
        k_m = budget // m + 1
        cell_id = np.arange(cells.shape[0])
        for n in avg_kernels:
            pooled = avg_pool_same(cells, int(n))
            order = np.lexsort((cell_id, -pooled.astype(np.float64)))[:k_m]
            added = 0
            for p in order:
                if added >= shares[combo]:
                    break
                for t in range(p * m, p * m + m):
                    if added >= shares[combo]:
                        break
                    if not allocated[t]:
                        allocated[t] = True
                        added += 1
            combo += 1
    return np.concatenate([np.arange(sink), sink + np.flatnonzero(allocated)]).astype(np.int64)


def thresholds_max_avg(score: np.ndarray, max_kernels: Sequence[int], avg_kernels: Sequence[int], budget: int,
                       sink: int = 0):
    """For the index-set comparison rule: replay allocate_max_avg and report, per combination, the pooled
    value of every token (its cell's average; NaN for the sink part and for tokens after the last whole
    cell), the value of the last cell that gave the combination a token (None if it took nothing) and the
    value of the K_m-th ranked cell (None if every cell is a candidate)."""
    L = score.shape[0]
    body = score[sink:]
    Lb = body.shape[0]
    shares = split_budget(budget, len(max_kernels) * len(avg_kernels))
    allocated = np.zeros(Lb, dtype=bool)
    out = []
    combo = 0
    for m in max_kernels:
        m = int(m)
        cells = max_pool_strided(body, m)
        k_m = budget // m + 1
        cell_id = np.arange(cells.shape[0])
        for n in avg_kernels:
            pooled = avg_pool_same(cells, int(n))
            ranked = np.lexsort((cell_id, -pooled.astype(np.float64)))
            order = ranked[:k_m]
            per_token = np.full(L, np.nan)
            per_token[sink:sink + cells.shape[0] * m] = np.repeat(pooled.astype(np.float64), m)
            added, last = 0, None
            for p in order:
                if added >= shares[combo]:
                    break
                for t in range(p * m, p * m + m):
                    if added >= shares[combo]:
                        break
                    if not allocated[t]:
                        allocated[t] = True
                        added += 1
                        last = float(pooled[p])
            cap = float(pooled[ranked[k_m - 1]]) if k_m < cells.shape[0] else None
            out.append((per_token, last, cap))
            combo += 1
    return out
