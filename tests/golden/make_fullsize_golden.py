#!/usr/bin/env python3
"""Writes tests/golden/fullsize_cfg{N}.json from the CPU oracle alone (imports only inputs/ and oracle/).

For the workloads too large for the oracle to run inside a GPU test, the oracle is run once here and
a compact digest is stored: sampled softmax row statistics, sampled per-token scores, the score total,
the recalled index set, each kernel's admission threshold and the tokens the comparison rule excuses
(oracle pooled score within 2*(1e-6 + 1e-3*thr_j) of a threshold), and the same pair (index set, excused
tokens) for Algorithm 1 as printed with the paper's default pooling set.  Usage:

    python tests/golden/make_fullsize_golden.py 3 4 5
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
N_ROWS, N_RANDOM_TOKENS, N_SELECTED_TOKENS = 256, 1024, 1024
PAPER_MAX, PAPER_AVG, PAPER_SINK = (2, 4, 8), tuple(range(1, 17)), 4   # default pooling set and sink size of the paper


def digest(cfg: int) -> dict:
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
    rng = np.random.default_rng(3000 + cfg)
    rows = np.sort(rng.choice(wl.Hq * wl.Lq, size=N_ROWS, replace=False))
    toks = np.unique(np.concatenate([rng.choice(wl.L, size=N_RANDOM_TOKENS, replace=False),
                                     rng.choice(idx, size=min(N_SELECTED_TOKENS, idx.size), replace=False)]))
    mask = inp.needle_mask
    near = np.zeros(wl.L, dtype=bool)                      # within 15 positions of a span
    for s, n in inp.spans:
        near[max(0, s - 15):min(wl.L, s + n + 15)] = True
    return {
        "cite": "Section 3.2, Eq. 4 / Eq. 5 (sum reading) / Algorithm 1 (stride-1 max-pool reading); written by "
                "tests/golden/make_fullsize_golden.py from oracle/ on inputs/ workload " + wl.name,
        "workload": wl.name, "cfg": cfg, "L": wl.L, "Lq": wl.Lq, "Hq": wl.Hq, "Hkv": wl.Hkv, "d": wl.d,
        "pool_kernels": list(wl.pool_kernels), "budget": wl.budget,
        "oracle_seconds": round(seconds, 1), "oracle_threads": oracle.num_threads(),
        "score_total": float(score.sum()),
        "rows": rows.tolist(),
        "row_max": [float(x) for x in rmax[rows]],
        "row_sumexp": [float(x) for x in rsum[rows]],
        "tokens": toks.tolist(),
        "token_scores": [float(x) for x in score[toks]],
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


def main() -> None:
    for cfg in [int(a) for a in sys.argv[1:]] or [3, 4, 5]:
        d = digest(cfg)
        path = os.path.join(ROOT, "tests", "golden", f"fullsize_cfg{cfg}.json")
        with open(path, "w") as f:
            json.dump(d, f, separators=(",", ":"))
            f.write("\n")
        print(f"cfg {cfg}: oracle {d['oracle_seconds']} s on {d['oracle_threads']} threads, total {d['score_total']:.6f}, "
              f"{len(d['excused_tokens'])} excusable tokens, needle recall {d['needle_recall']:.3f}, "
              f"precision {d['precision_within_15_of_a_span']:.3f} -> {path}", flush=True)


if __name__ == "__main__":
    main()
