#!/usr/bin/env python3
"""Writes the full-size expected values of tests/golden/ from the CPU oracle alone (imports only inputs/
and oracle/).

For the workloads too large for the oracle to run inside a GPU test (cfg 4: 512K tokens, cfg 5: 1M tokens),
the oracle is run once here and everything the GPU test compares is stored, nothing sampled:

    fullsize_cfg{N}_scores.npy     the oracle's per-token score of Eq. 5, all L of them, rounded to float32
                                   (a relative 6e-8 against the 1e-3 the comparison allows)
    fullsize_cfg{N}_rowstats.npy   float64 [2, Hq*Lq]: row maximum and sum of exponentials of Eq. 4, every row
    fullsize_cfg{N}.json           shape, oracle wall time and thread count, the score total, and for both
                                   forms of Algorithm 1 the recalled index set, each kernel's admission
                                   threshold and the tokens the comparison rule excuses (oracle pooled score
                                   within 2*(1e-6 + 1e-3*thr_j) of a threshold)

Usage:    python tests/golden/make_fullsize_golden.py 4 5
"""
from __future__ import annotations

import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import inputs  # noqa: E402
import oracle  # noqa: E402

REL_TOL, ABS_TOL = 1e-3, 1e-6
PAPER_MAX, PAPER_AVG, PAPER_SINK = (2, 4, 8), tuple(range(1, 17)), 4   # default pooling set and sink size of the paper


def digest(cfg: int):
    wl = inputs.CONFIGS[cfg]
    inp = inputs.generate(wl)
    t0 = time.time()
    score, rmax, rsum = oracle.scores(inp.q, inp.k)
    seconds = time.time() - t0
    s32 = score.astype(np.float32)
    idx = oracle.allocate(s32, wl.pool_kernels, wl.budget)
    th = oracle.thresholds(s32, wl.pool_kernels, wl.budget)
    excused = np.zeros(wl.L, dtype=bool)
    thr_list = []
    for pooled, thr in th:
        thr_list.append(thr)
        if thr is not None:
            excused |= np.abs(pooled.astype(np.float64) - thr) <= 2 * (ABS_TOL + REL_TOL * abs(thr))
    # Algorithm 1 as printed on the same scores: index set and the tokens its comparison rule excuses
    # (cell average within tolerance of what a combination last admitted or of its K_m-th ranked cell)
    ma_idx = oracle.allocate_max_avg(s32, PAPER_MAX, PAPER_AVG, wl.budget, sink=PAPER_SINK)
    ma_excused = np.zeros(wl.L, dtype=bool)
    for per_token, last, cap in oracle.thresholds_max_avg(s32, PAPER_MAX, PAPER_AVG, wl.budget, sink=PAPER_SINK):
        for thr in (last, cap):
            if thr is not None:
                with np.errstate(invalid="ignore"):
                    ma_excused |= np.abs(per_token - thr) <= 2 * (ABS_TOL + REL_TOL * abs(thr))
    mask = inp.needle_mask
    near = np.zeros(wl.L, dtype=bool)                      # within 15 positions of a span
    for s, n in inp.spans:
        near[max(0, s - 15):min(wl.L, s + n + 15)] = True
    meta = {
        "cite": "Section 3.2, Eq. 4 / Eq. 5 (sum reading) / Algorithm 1 (stride-1 max-pool reading and as printed); "
                "written by tests/golden/make_fullsize_golden.py from oracle/ on inputs/ workload " + wl.name,
        "workload": wl.name, "cfg": cfg, "L": wl.L, "Lq": wl.Lq, "Hq": wl.Hq, "Hkv": wl.Hkv, "d": wl.d,
        "pool_kernels": list(wl.pool_kernels), "budget": wl.budget,
        "oracle_seconds": round(seconds, 1), "oracle_threads": oracle.num_threads(),
        "score_total": float(score.sum()),
        "indices": idx.tolist(),
        "thresholds": thr_list,
        "excused_tokens": np.flatnonzero(excused).tolist(),
        "max_avg": {"max_kernels": list(PAPER_MAX), "avg_kernels": list(PAPER_AVG), "sink": PAPER_SINK,
                    "indices": ma_idx.tolist(), "excused_tokens": np.flatnonzero(ma_excused).tolist(),
                    "needle_recall": float(mask[ma_idx].sum() / max(1, mask.sum()))},
        "needle_tokens": int(mask.sum()),
        "needle_recall": float(mask[idx].sum() / max(1, mask.sum())),
        "precision_within_15_of_a_span": float(near[idx].mean()),
    }
    return meta, s32, np.stack([rmax, rsum])


def main() -> None:
    gdir = os.path.join(ROOT, "tests", "golden")
    for cfg in [int(a) for a in sys.argv[1:]] or [4, 5]:
        d, s32, rowstats = digest(cfg)
        path = os.path.join(gdir, f"fullsize_cfg{cfg}.json")
        with open(path, "w") as f:
            json.dump(d, f, separators=(",", ":"))
            f.write("\n")
        np.save(os.path.join(gdir, f"fullsize_cfg{cfg}_scores.npy"), s32)
        np.save(os.path.join(gdir, f"fullsize_cfg{cfg}_rowstats.npy"), rowstats)
        print(f"cfg {cfg}: oracle {d['oracle_seconds']} s on {d['oracle_threads']} threads, total {d['score_total']:.6f}, "
              f"{len(d['excused_tokens'])} excusable tokens, needle recall {d['needle_recall']:.3f}, "
              f"precision {d['precision_within_15_of_a_span']:.3f} -> {path}", flush=True)


if __name__ == "__main__":
    main()
