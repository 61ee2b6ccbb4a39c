"""Plain fp64 CPU oracle of the token-recall path.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this package; it
shares no code with the GPU path and never imports it.
"""
from __future__ import annotations

import numpy as np

from .allocation import (allocate, allocate_max_avg, avg_pool_same, max_pool_same, max_pool_strided, split_budget,
                         thresholds, thresholds_max_avg)
from .rerope import PAIR_HALF, PAIR_INTERLEAVED, chunk_bounds, chunk_distances, default_inv_freq, rerope_keys, rotate
from .scoring import MODE_MAX, MODE_SUM, num_threads, row_stats, scores


def recall(q, k, pool_kernels, budget, scale=None, mode=MODE_SUM):
    """Whole path: Eq. 4, Eq. 5, then Algorithm 1 decided on the fp32-rounded scores (the
    precision the GPU path decides in).  Returns (indices int64 ascending, score fp64[L])."""
    score, _, _ = scores(q, k, scale=scale, mode=mode)
    idx = allocate(score.astype(np.float32), pool_kernels, budget)
    return idx, score


def recall_max_avg(q, k, max_kernels, avg_kernels, budget, sink=0, scale=None, mode=MODE_SUM):
    """Whole path with Algorithm 1 as printed: Eq. 4 over all positions (the sink part included), Eq. 5,
    then the allocation decided on the fp32-rounded scores.  Returns (indices int64 ascending, score fp64[L])."""
    score, _, _ = scores(q, k, scale=scale, mode=mode)
    idx = allocate_max_avg(score.astype(np.float32), max_kernels, avg_kernels, budget, sink=sink)
    return idx, score


__all__ = ["rerope_keys", "rotate", "chunk_bounds", "chunk_distances", "default_inv_freq", "PAIR_HALF", "PAIR_INTERLEAVED", "recall_max_avg", "thresholds_max_avg", "allocate", "allocate_max_avg", "avg_pool_same", "max_pool_strided", "max_pool_same", "split_budget", "thresholds", "scores", "row_stats",
           "num_threads", "recall", "MODE_SUM", "MODE_MAX"]
