"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times (one
ilre_recall call on the generated workload).  The oracle cannot run these sizes inside a test, so
the expected values are the digests written from oracle/ by tests/golden/make_fullsize_golden.py:
sampled row statistics, sampled scores, the score total, the recalled index set and the tokens the
threshold rule excuses."""
import json
import os

import numpy as np
import pytest
import torch

import inputs
import paper_2508_17892_amd as il
from parity import check_index_structure, score_errors, to_device

pytestmark = pytest.mark.gpu


def _load(golden_dir, cfg):
    path = os.path.join(golden_dir, f"fullsize_cfg{cfg}.json")
    if not os.path.exists(path):
        pytest.skip(f"{path} not generated")
    with open(path) as f:
        return json.load(f)


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_fullsize_against_oracle_digest(cfg, golden_dir):
    g = _load(golden_dir, cfg)
    print(f"[case] fullsize cfg{cfg} L={g['L']} Lq={g['Lq']}", flush=True)
    wl = inputs.CONFIGS[cfg]
    assert (wl.L, wl.Lq, wl.Hq, wl.Hkv, list(wl.pool_kernels), wl.budget) == \
        (g["L"], g["Lq"], g["Hq"], g["Hkv"], g["pool_kernels"], g["budget"])
    inp = inputs.generate(wl)
    q, k = to_device(inp.q), to_device(inp.k)
    del inp
    ws = il.alloc_workspace(wl.L, wl.Lq, wl.Hq, wl.Hkv, wl.d, len(wl.pool_kernels), il.ILRE_BF16)
    idx, scores = il.ilre_recall(q, k, wl.budget, wl.pool_kernels, workspace=ws)
    row_max, row_sumexp = il.ilre_row_stats(q, k, workspace=ws)
    torch.cuda.synchronize()
    idx, scores = idx.cpu().numpy(), scores.cpu().numpy()

    # softmax row statistics on the sampled rows: the (reference, sum) pair encodes the oracle's
    # log-sum-exp; with the exact-maximum flag the pair itself matches (checked at the smallest size)
    rows = np.array(g["rows"])
    want_lse = np.array(g["row_max"]) + np.log(np.array(g["row_sumexp"]))
    got_lse = row_max.cpu().numpy()[rows].astype(np.float64) + np.log(row_sumexp.cpu().numpy()[rows].astype(np.float64))
    np.testing.assert_allclose(got_lse, want_lse, rtol=0, atol=2e-4)
    if cfg == 3:
        em, ez = il.ilre_row_stats(q, k, workspace=ws, flags=il.ILRE_FLAG_EXACT_ROW_MAX)
        np.testing.assert_allclose(em.cpu().numpy()[rows].astype(np.float64), np.array(g["row_max"]), rtol=0, atol=1e-4)
        np.testing.assert_allclose(ez.cpu().numpy()[rows].astype(np.float64), np.array(g["row_sumexp"]), rtol=2e-4)

    # per-token scores on the sampled tokens; total mass = number of softmax rows
    toks = np.array(g["tokens"])
    bad, worst = score_errors(scores[toks], np.array(g["token_scores"]))
    assert bad == 0, f"{bad} of {toks.size} sampled scores out of tolerance, worst {worst:.2f}x"
    total = float(scores.astype(np.float64).sum())
    assert abs(total - wl.Hq * wl.Lq) < 1e-4 * wl.Hq * wl.Lq
    assert abs(g["score_total"] - wl.Hq * wl.Lq) < 1e-6 * wl.Hq * wl.Lq

    # recalled index set: identical up to the tokens within tolerance of a kernel's threshold
    check_index_structure(idx, wl.L, wl.budget)
    diff = set(idx.tolist()) ^ set(g["indices"])
    unexcused = sorted(diff - set(g["excused_tokens"]))
    assert not unexcused, f"{len(unexcused)} unexcused index differences, e.g. {unexcused[:8]}"
    print(f"[case] fullsize cfg{cfg}: worst score error {worst:.3f} of tolerance, index sym diff {len(diff)} (all excused)",
          flush=True)


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_fullsize_printed_allocation_against_oracle_digest(cfg, golden_dir):
    """Algorithm 1 as printed (the paper's default pooling set, sink 4) on the full-size workloads:
    index set equal to the oracle's up to the tokens its threshold rule excuses."""
    g = _load(golden_dir, cfg)
    if "max_avg" not in g:
        pytest.skip("digest written before the printed form was added")
    ma = g["max_avg"]
    print(f"[case] fullsize printed allocation cfg{cfg} L={g['L']}", flush=True)
    wl = inputs.CONFIGS[cfg]
    inp = inputs.generate(wl)
    q, k = to_device(inp.q), to_device(inp.k)
    del inp
    idx, count, scores = il.ilre_recall_max_avg(q, k, wl.budget, ma["max_kernels"], ma["avg_kernels"], ma["sink"])
    torch.cuda.synchronize()
    n = int(count.item())
    idx = idx.cpu().numpy()
    assert (idx[n:] == -1).all() and (np.diff(idx[:n].astype(np.int64)) > 0).all()
    assert idx[:ma["sink"]].tolist() == list(range(ma["sink"]))
    toks = np.array(g["tokens"])
    bad, worst = score_errors(scores.cpu().numpy()[toks], np.array(g["token_scores"]))
    assert bad == 0, worst
    diff = set(idx[:n].tolist()) ^ set(ma["indices"])
    unexcused = sorted(diff - set(ma["excused_tokens"]))
    assert not unexcused, f"{len(unexcused)} unexcused index differences, e.g. {unexcused[:8]}"
    print(f"[case] fullsize printed allocation cfg{cfg}: kept {n}, index sym diff {len(diff)} (all excused)", flush=True)
