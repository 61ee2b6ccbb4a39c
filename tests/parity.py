"""Comparison rules shared by the GPU parity tests, the smoke check and the benchmark.

Scores: |gpu - oracle| <= ABS_TOL + REL_TOL * |oracle| for every token.
Index sets: identical, except that a token in the symmetric difference is excused when, for some
pooling kernel j, its oracle pooled score lies within 2*(ABS_TOL + REL_TOL*thr_j) of the pooled
score thr_j of the last token that kernel admitted in the oracle's run.
"""
from __future__ import annotations

import numpy as np

import oracle
from paper_2508_17892_amd import to_device  # noqa: F401  (re-exported for the GPU tests)

REL_TOL = 1e-3
ABS_TOL = 1e-6


def score_errors(gpu_scores: np.ndarray, oracle_scores: np.ndarray):
    """Returns (number of tokens out of tolerance, worst error / allowed error)."""
    err = np.abs(gpu_scores.astype(np.float64) - oracle_scores)
    allowed = ABS_TOL + REL_TOL * np.abs(oracle_scores)
    return int((err > allowed).sum()), float((err / allowed).max())


def index_set_report(gpu_idx: np.ndarray, oracle_scores: np.ndarray, pool_kernels, budget: int):
    """Returns dict(sym_diff, excused, unexcused list).  Decisions on the oracle side are taken on its
    scores rounded to float32, the precision the GPU path decides in."""
    s32 = oracle_scores.astype(np.float32)
    want = oracle.allocate(s32, pool_kernels, budget)
    g = set(int(x) for x in gpu_idx.tolist())
    o = set(int(x) for x in want.tolist())
    diff = sorted(g ^ o)
    unexcused = []
    if diff:
        th = oracle.thresholds(s32, pool_kernels, budget)
        for t in diff:
            ok = False
            for pooled, thr in th:
                if thr is None:
                    continue
                if abs(float(pooled[t]) - thr) <= 2 * (ABS_TOL + REL_TOL * abs(thr)):
                    ok = True
                    break
            if not ok:
                unexcused.append(t)
    return {"sym_diff": len(diff), "excused": len(diff) - len(unexcused), "unexcused": unexcused,
            "n_gpu": len(gpu_idx), "n_oracle": len(want)}


def index_set_report_max_avg(gpu_idx: np.ndarray, oracle_scores: np.ndarray, max_kernels, avg_kernels, budget: int,
                             sink: int):
    """The same rule for Algorithm 1 as printed: a token in the symmetric difference is excused when, for
    some combination, the oracle's average of its cell lies within 2*(ABS_TOL + REL_TOL*thr) of thr = the value
    of the last cell that combination admitted from, or of its K_m-th ranked cell (the candidate cap)."""
    s32 = oracle_scores.astype(np.float32)
    want = oracle.allocate_max_avg(s32, max_kernels, avg_kernels, budget, sink=sink)
    g = set(int(x) for x in gpu_idx.tolist())
    o = set(int(x) for x in want.tolist())
    diff = sorted(g ^ o)
    unexcused = []
    if diff:
        th = oracle.thresholds_max_avg(s32, max_kernels, avg_kernels, budget, sink=sink)
        for t in diff:
            ok = False
            for per_token, last, cap in th:
                v = per_token[t]
                if np.isnan(v):
                    continue
                for thr in (last, cap):
                    if thr is not None and abs(v - thr) <= 2 * (ABS_TOL + REL_TOL * abs(thr)):
                        ok = True
            if not ok:
                unexcused.append(t)
    return {"sym_diff": len(diff), "excused": len(diff) - len(unexcused), "unexcused": unexcused,
            "n_gpu": len(gpu_idx), "n_oracle": len(want)}


def check_index_structure(idx: np.ndarray, L: int, budget: int):
    assert idx.shape == (min(budget, L),)
    assert idx.dtype == np.int32
    assert (np.diff(idx.astype(np.int64)) > 0).all(), "indices must be strictly ascending"
    assert idx.min() >= 0 and idx.max() < L
