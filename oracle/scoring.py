"""ctypes front of the C scoring oracle (Eq. 4 and Eq. 5 of the paper, Section 3.2).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
cpu_baseline leg.  The product path never calls it.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None

MODE_SUM, MODE_MAX = 0, 1


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        lib = ctypes.CDLL(path)
        i64, i32, dbl, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.c_void_p
        lib.ilre_oracle_scores.restype = ctypes.c_int
        lib.ilre_oracle_scores.argtypes = [vp, vp, ctypes.c_int, i64, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_int, ctypes.c_int, dbl, ctypes.c_int, vp, vp, vp]
        lib.ilre_oracle_row_stats.restype = ctypes.c_int
        lib.ilre_oracle_row_stats.argtypes = [vp, vp, ctypes.c_int, i64, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_int, ctypes.c_int, dbl, vp, ctypes.c_int, vp, vp]
        lib.ilre_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _prep(q: np.ndarray, k: np.ndarray):
    if q.dtype != k.dtype or q.dtype not in (np.dtype(np.float32), np.dtype(np.uint16)):
        raise TypeError("q and k must both be float32, or both uint16 bf16 bit patterns")
    if q.ndim != 3 or k.ndim != 3 or q.shape[2] != k.shape[2]:
        raise ValueError("q is [Hq, Lq, d], k is [Hkv, L, d]")
    q = np.ascontiguousarray(q)
    k = np.ascontiguousarray(k)
    Hq, Lq, d = q.shape
    Hkv, L, _ = k.shape
    if Hq % Hkv:
        raise ValueError("Hq must be a multiple of Hkv")
    dtype = 1 if q.dtype == np.uint16 else 0
    return q, k, dtype, L, Lq, Hq, Hkv, d


def num_threads() -> int:
    return int(_load().ilre_oracle_num_threads())


def scores(q: np.ndarray, k: np.ndarray, scale: float | None = None, mode: int = MODE_SUM):
    """Per-token score (Eq. 4 then Eq. 5) plus the softmax row statistics, all fp64.

    Returns (score[L], row_max[Hq*Lq], row_sumexp[Hq*Lq]); row r = h*Lq + i.
    """
    q, k, dtype, L, Lq, Hq, Hkv, d = _prep(q, k)
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    score = np.empty(L, dtype=np.float64)
    rmax = np.empty(Hq * Lq, dtype=np.float64)
    rsum = np.empty(Hq * Lq, dtype=np.float64)
    rc = _load().ilre_oracle_scores(q.ctypes.data, k.ctypes.data, dtype, L, Lq, Hq, Hkv, d, scale, mode,
                                    rmax.ctypes.data, rsum.ctypes.data, score.ctypes.data)
    if rc != 0:
        raise RuntimeError("ilre_oracle_scores failed")
    return score, rmax, rsum


def row_stats(q: np.ndarray, k: np.ndarray, rows, scale: float | None = None):
    """Softmax row maximum and sum of exponentials (Eq. 4) for the listed rows r = h*Lq + i."""
    q, k, dtype, L, Lq, Hq, Hkv, d = _prep(q, k)
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    if rows.size and (rows.min() < 0 or rows.max() >= Hq * Lq):
        raise ValueError("row index out of range")
    rmax = np.empty(rows.size, dtype=np.float64)
    rsum = np.empty(rows.size, dtype=np.float64)
    rc = _load().ilre_oracle_row_stats(q.ctypes.data, k.ctypes.data, dtype, L, Lq, Hq, Hkv, d, scale,
                                       rows.ctypes.data, rows.size, rmax.ctypes.data, rsum.ctypes.data)
    if rc != 0:
        raise RuntimeError("ilre_oracle_row_stats failed")
    return rmax, rsum
