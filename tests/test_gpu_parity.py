"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Staged (row statistics, column scores, selection) and end to end."""
import zlib

import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2508_17892_amd as il
from parity import (ABS_TOL, REL_TOL, check_index_structure, index_set_report, index_set_report_max_avg, score_errors,
                    to_device)

pytestmark = pytest.mark.gpu


def _announce(msg):
    print(f"[case] {msg}", flush=True)


SHAPES = [
    # name, L, Lq, Hq, Hkv, dtype, channel_scale
    ("bf16_ragged_small", 1000, 8, 8, 2, "bf16", False),       # 32 rows/group: mostly padded rows, ragged tail
    ("bf16_multi_tile", 5000, 64, 8, 2, "bf16", True),         # 256 rows/group: 4-wave workgroups
    ("bf16_two_query_blocks", 3333, 160, 8, 1, "bf16", True),  # 1280 rows/group: 8-wave workgroups, 3 query blocks
    ("f32_small", 777, 32, 8, 2, "f32", False),
    ("f32_two_query_blocks", 2100, 48, 8, 2, "f32", True),     # 192 rows/group: 2 query blocks of 128
    ("bf16_single_token", 1, 4, 4, 2, "bf16", False),
    ("bf16_exact_tiles", 4096, 32, 32, 8, "bf16", False),
    # head counts of the other models the paper evaluates (Section 4): GQA groups of 7 and of 8
    ("qwen2_5_7b_heads", 3000, 64, 28, 4, "bf16", True),       # 448 rows/group: one 8-wave query block, 64 rows padded
    ("qwen3_32b_heads", 2500, 40, 64, 8, "bf16", True),        # 320 rows/group: two 4-wave query blocks
]


@pytest.mark.parametrize("name,L,Lq,Hq,Hkv,dtype,cs", SHAPES, ids=[s[0] for s in SHAPES])
def test_staged_scoring(name, L, Lq, Hq, Hkv, dtype, cs):
    _announce(f"staged_scoring {name} L={L} Lq={Lq} Hq={Hq} Hkv={Hkv} {dtype}")
    inp = inputs.custom(L=L, Lq=Lq, Hq=Hq, Hkv=Hkv, d=128, dtype=dtype, n_spans=2 if L > 200 else 0,
                        span_len=(8, 24), channel_scale=cs, seed=zlib.crc32(name.encode()) % 1000)
    q, k = to_device(inp.q), to_device(inp.k)
    want_score, want_max, want_sum = oracle.scores(inp.q, inp.k)

    # exact form: the reference is the row maximum itself
    row_max, row_sumexp = il.ilre_row_stats(q, k, flags=il.ILRE_FLAG_EXACT_ROW_MAX)
    torch.cuda.synchronize()
    gm, gz = row_max.cpu().numpy().astype(np.float64), row_sumexp.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(gm, want_max, rtol=0, atol=1e-4)
    np.testing.assert_allclose(gz, want_sum, rtol=2e-4)
    # default form: a reference at or below the maximum, same log-sum-exp
    row_max, row_sumexp = il.ilre_row_stats(q, k)
    torch.cuda.synchronize()
    gm, gz = row_max.cpu().numpy().astype(np.float64), row_sumexp.cpu().numpy().astype(np.float64)
    assert (gm <= want_max + 1e-4).all() and np.isfinite(gz).all() and (gz >= 1.0 - 1e-5).all()
    np.testing.assert_allclose(gm + np.log(gz), want_max + np.log(want_sum), rtol=0, atol=2e-4)

    got = il.ilre_col_scores(q, k, row_max, row_sumexp)
    torch.cuda.synchronize()
    bad, worst = score_errors(got.cpu().numpy(), want_score)
    assert bad == 0, f"{bad} scores out of tolerance, worst {worst:.2f}x"
    assert abs(float(got.double().sum()) - Hq * Lq) < 1e-3 * Hq * Lq

    # column scores from the oracle's own row statistics (stage isolation)
    got2 = il.ilre_col_scores(q, k, torch.from_numpy(want_max.astype(np.float32)).cuda(),
                              torch.from_numpy(want_sum.astype(np.float32)).cuda())
    bad, worst = score_errors(got2.cpu().numpy(), want_score)
    assert bad == 0, f"{bad} scores out of tolerance, worst {worst:.2f}x"

    # Eq. 5 as printed: max over heads and queries
    want_mx, _, _ = oracle.scores(inp.q, inp.k, mode=oracle.MODE_MAX)
    got_mx = il.ilre_col_scores(q, k, row_max, row_sumexp, score_mode=il.ILRE_SCORE_MAX)
    bad, worst = score_errors(got_mx.cpu().numpy(), want_mx)
    assert bad == 0, f"max mode: {bad} scores out of tolerance, worst {worst:.2f}x"


@pytest.mark.parametrize("seed", range(3))
def test_scoring_randomised_shapes(seed):
    """Random shapes around the kernels' block sizes (32-row query blocks, 64/128-token tiles, 4- and 8-wave
    workgroups, several token splits), both element types, sum and max reduction, whole path."""
    _announce(f"randomised scoring shapes, seed {seed}")
    rng = np.random.default_rng(7000 + seed)
    for case in range(6):
        Hkv = int(rng.choice([1, 2, 3]))
        G = int(rng.choice([1, 2, 4, 5]))
        Lq = int(rng.choice([1, 7, 31, 33, 64, 100, 130]))
        L = int(rng.choice([1, 31, 64, 127, 129, 1000, 4097, 12000])) + int(rng.integers(0, 3))
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        inp = inputs.custom(L=L, Lq=Lq, Hq=Hkv * G, Hkv=Hkv, d=128, dtype=dtype, n_spans=1 if L > 300 else 0,
                            span_len=(8, 24), channel_scale=bool(rng.integers(2)), seed=100 * seed + case)
        q, k = to_device(inp.q), to_device(inp.k)
        mode = oracle.MODE_MAX if case % 3 == 2 else oracle.MODE_SUM
        want, _, _ = oracle.scores(inp.q, inp.k, mode=mode)
        _, got = il.ilre_recall(q, k, 16, (3,), score_mode=il.ILRE_SCORE_MAX if mode == oracle.MODE_MAX else il.ILRE_SCORE_SUM)
        torch.cuda.synchronize()
        bad, worst = score_errors(got.cpu().numpy(), want)
        assert bad == 0, (seed, case, L, Lq, Hkv, G, dtype, mode, bad, worst)


SELECT_CASES = [
    # name, L, kernels, budget, kind
    ("random_small", 3000, (3, 7, 15), 256, "random"),
    ("random_multi_chunk", 50000, (1, 3, 7, 15, 31), 4096, "random"),
    ("plateaus", 20000, (3, 7, 15, 31), 1024, "few_values"),
    ("all_equal", 10000, (3, 7, 15), 100, "equal"),
    ("budget_exceeds_L", 300, (3, 7), 1000, "random"),
    ("L_smaller_than_kernel", 9, (31, 15), 4, "random"),
    ("budget_not_divisible", 7000, (3, 7, 15), 256, "random"),
    ("budget_below_kernel_count", 500, (1, 3, 5, 7), 3, "random"),
    ("single_token", 1, (3,), 1, "random"),
    ("wide_kernel", 30000, (2047, 1, 255), 600, "random"),
    ("needle_like", 100000, (1, 3, 7, 15, 31), 4096, "needles"),
    ("dense_background_ties", 200000, (3, 7, 15, 31), 4096, "narrow"),
    ("max_budget", 40000, (3, 31), 8192, "random"),
    ("twelve_kernels_two_groups", 30000, (1, 3, 5, 7, 9, 11, 13, 15, 31, 63, 127, 3), 3000, "needles"),
    ("all_equal_large", 300000, (3, 7, 15, 31), 4096, "equal"),
    ("two_values_heavy_ties", 150000, (1, 7), 5000, "two_values"),
    # a later list whose best tokens are all taken: the walk has to go past its first stretch of ranks
    ("repeated_kernel_sizes", 60000, (7, 7, 7, 7), 2000, "random"),
    ("small_after_large", 80000, (63, 3, 1), 3000, "needles"),
    # long contexts: the pruning pre-pass (fine-chunk maxima) decides which chunks are visited
    ("pruned_needles", 5000000, (1, 3, 7, 15, 31), 4096, "needles"),
    ("pruned_dense_background", 4500001, (3, 31), 1000, "narrow"),
    ("pruned_wide_kernel", 5000000, (511, 3), 500, "needles"),
    ("pruned_all_equal", 4200000, (3, 7), 64, "equal"),
]


def _scores_for(kind, L, rng):
    if kind == "random":
        return rng.random(L).astype(np.float32)
    if kind == "few_values":
        return (rng.integers(1, 9, size=L) / 16.0).astype(np.float32)
    if kind == "two_values":
        return np.where(rng.random(L) < 0.01, 0.5, 0.25).astype(np.float32)
    if kind == "equal":
        return np.full(L, 0.125, dtype=np.float32)
    if kind == "narrow":   # a dense background inside one binade, as real scores are
        return (0.0078125 * (1.0 + 0.5 * rng.random(L))).astype(np.float32)
    s = (0.008 * (1.0 + 0.3 * rng.standard_normal(L))).clip(1e-4).astype(np.float32)
    for start in rng.integers(0, L - 300, size=20):
        n = int(rng.integers(64, 256))
        s[start:start + n] = (rng.random(n) * 8).astype(np.float32)
    return s


@pytest.mark.parametrize("name,L,kernels,budget,kind", SELECT_CASES, ids=[c[0] for c in SELECT_CASES])
def test_select_exact_on_given_scores(name, L, kernels, budget, kind):
    _announce(f"select {name} L={L} kernels={kernels} budget={budget}")
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    s = _scores_for(kind, L, rng)
    want = oracle.allocate(s, kernels, budget)
    got = il.ilre_select(torch.from_numpy(s).cuda(), budget, kernels)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    check_index_structure(got, L, budget)
    assert got.tolist() == want.tolist()


SINK_CASES = [
    # name, L, sink, kernels, budget, kind
    ("paper_sink_needles", 100000, 4, (1, 3, 7, 15, 31), 4096, "needles"),
    ("sink_scores_dominate", 20000, 5, (3, 7, 15), 1000, "random"),
    ("sink_is_everything", 37, 37, (3,), 16, "random"),
    ("sink_leaves_one_token", 38, 37, (3, 7), 16, "random"),
    ("sink_and_budget_exceed_L", 300, 4, (3, 7), 1000, "random"),
    ("sink_all_equal", 10000, 3, (3, 7, 15), 100, "equal"),
    ("sink_pruned_long_context", 4500001, 4, (1, 3, 7, 15, 31), 4096, "needles"),
]


@pytest.mark.parametrize("name,L,sink,kernels,budget,kind", SINK_CASES, ids=[c[0] for c in SINK_CASES])
def test_select_with_a_sink_part(name, L, sink, kernels, budget, kind):
    """Window-max form with the sink part of Algorithm 1: the first `sink` tokens always kept and invisible to
    the pooling (their scores are set far above everything else, so any leak would show), the budget counting
    the others; bit-exact with the oracle."""
    _announce(f"select with sink {name} L={L} sink={sink} kernels={kernels} budget={budget}")
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    s = _scores_for(kind, L, rng) if L > 300 else rng.random(L).astype(np.float32)
    s[:sink] = 1000.0
    want = oracle.allocate(s, kernels, budget, sink=sink)
    got = il.ilre_select(torch.from_numpy(s).cuda(), budget, kernels, sink=sink)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert got.shape == (sink + min(budget, L - sink),) and got.dtype == np.int32
    assert got.tolist() == want.tolist()


def test_recall_with_a_sink_part():
    """Whole path with a sink part: same scores as without (Eq. 4 runs over all L positions), selection equal to
    the staged call and to the oracle's Algorithm 1 on the GPU's own scores."""
    _announce("end_to_end with sink 4 (ragged bf16)")
    inp = inputs.custom(L=9001, Lq=40, Hq=16, Hkv=4, d=128, dtype="bf16", n_spans=3, span_len=(16, 40),
                        channel_scale=True, seed=78)
    q, k = to_device(inp.q), to_device(inp.k)
    kernels, budget, sink = (1, 3, 7, 15, 31), 512, 4
    idx, scores = il.ilre_recall(q, k, budget, kernels, sink=sink)
    _, plain_scores = il.ilre_recall(q, k, budget, kernels)
    staged = il.ilre_select(scores, budget, kernels, sink=sink)
    torch.cuda.synchronize()
    assert torch.equal(scores, plain_scores) and torch.equal(idx, staged)
    assert idx.cpu().numpy().tolist() == oracle.allocate(scores.cpu().numpy(), kernels, budget, sink=sink).tolist()
    want_scores, _, _ = oracle.scores(inp.q, inp.k)
    bad, worst = score_errors(scores.cpu().numpy(), want_scores)
    assert bad == 0, worst


PAPER_MAX, PAPER_AVG = (2, 4, 8), tuple(range(1, 17))     # the paper's default pooling set (Section 3.2)

MAX_AVG_CASES = [
    # name, L, sink, max kernels, avg kernels, budget, kind of scores
    ("paper_default_needles", 100000, 4, PAPER_MAX, PAPER_AVG, 4096, "needles"),
    ("paper_default_ragged", 50001, 4, PAPER_MAX, PAPER_AVG, 1024, "random"),
    ("snapkv_special_case", 30000, 0, (1,), (7,), 1000, "random"),
    ("plain_topk", 20000, 0, (1,), (1,), 512, "random"),
    ("one_max_avg", 40000, 4, (4,), (5,), 2048, "needles"),
    ("odd_max_kernels", 33333, 3, (3, 5, 6, 7), (1, 2, 3, 4, 9), 3000, "random"),
    ("candidates_exhausted", 3000, 2, (8, 8, 4), (1, 2, 3), 2500, "random"),
    ("budget_exceeds_L", 700, 4, (2, 4), (1, 3), 5000, "random"),
    ("budget_below_combination_count", 5000, 4, PAPER_MAX, PAPER_AVG, 5, "random"),
    ("all_equal", 60000, 4, PAPER_MAX, (1, 2, 5, 16), 4096, "equal"),
    ("plateaus", 70000, 0, (2, 8), (1, 4, 16), 4096, "few_values"),
    ("two_values_heavy_ties", 150000, 4, (2, 4), (1, 2), 6000, "two_values"),
    ("dense_background", 200000, 4, PAPER_MAX, PAPER_AVG, 4096, "narrow"),
    ("signed_with_zeros", 25000, 1, (2, 3), (1, 2, 6), 800, "signed"),
    ("wide_kernels", 90000, 0, (1024, 256), (1024, 33), 8192, "needles"),
    ("L_below_max_kernel", 5, 0, (8, 2), (1, 3), 4, "random"),
    ("sink_is_everything", 37, 37, (2,), (3,), 16, "random"),
    ("sink_leaves_one_token", 38, 37, (1, 2), (3,), 16, "random"),
    ("max_budget", 50000, 4, PAPER_MAX, PAPER_AVG, 8192, "random"),
    ("one_million_paper_default", 1 << 20, 4, PAPER_MAX, PAPER_AVG, 4096, "needles"),
]


@pytest.mark.parametrize("name,L,sink,mk,ak,budget,kind", MAX_AVG_CASES, ids=[c[0] for c in MAX_AVG_CASES])
def test_select_max_avg_exact_on_given_scores(name, L, sink, mk, ak, budget, kind):
    """Algorithm 1 as printed (strided max pooling, average pooling, K_m cap, sink part): bit-exact with
    the oracle on the same float32 scores, the unused tail of the output marked -1."""
    _announce(f"select_max_avg {name} L={L} sink={sink} max={mk} avg={ak} budget={budget}")
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    if kind == "signed":
        s = rng.standard_normal(L).astype(np.float32)
        s[rng.random(L) < 0.3] = 0.0
        s[rng.random(L) < 0.1] = -0.0
    else:
        s = _scores_for(kind, L, rng) if L > 300 else rng.random(L).astype(np.float32)
    want = oracle.allocate_max_avg(s, mk, ak, budget, sink=sink)
    got, count = il.ilre_select_max_avg(torch.from_numpy(s).cuda(), budget, mk, ak, sink)
    torch.cuda.synchronize()
    got, count = got.cpu().numpy(), int(count.item())
    assert got.shape == (sink + min(budget, L - sink),) and got.dtype == np.int32
    assert count == len(want)
    assert got[:count].tolist() == want.tolist()
    assert (got[count:] == -1).all()


def test_select_max_avg_reuses_a_workspace():
    """Two calls in a row on one workspace, the second smaller: nothing of the first leaks into it."""
    _announce("select_max_avg workspace reuse")
    rng = np.random.default_rng(11)
    big, small = _scores_for("needles", 80000, rng), rng.random(9000).astype(np.float32)
    ws = il.alloc_workspace_max_avg(80000, 1, 1, 1, 128, 4, PAPER_MAX, len(PAPER_AVG), il.ILRE_F32)
    for s, budget in ((big, 4096), (small, 700), (big, 4096)):
        want = oracle.allocate_max_avg(s, PAPER_MAX, PAPER_AVG, budget, sink=4)
        got, count = il.ilre_select_max_avg(torch.from_numpy(s).cuda(), budget, PAPER_MAX, PAPER_AVG, 4, workspace=ws)
        torch.cuda.synchronize()
        assert got.cpu().numpy()[:int(count.item())].tolist() == want.tolist()


def _end_to_end(inp, kernels, budget):
    wl = inp.workload
    q, k = to_device(inp.q), to_device(inp.k)
    idx, scores = il.ilre_recall(q, k, budget, kernels)
    torch.cuda.synchronize()
    idx, scores = idx.cpu().numpy(), scores.cpu().numpy()
    want_scores, _, _ = oracle.scores(inp.q, inp.k)
    bad, worst = score_errors(scores, want_scores)
    assert bad == 0, f"{bad} scores out of tolerance, worst {worst:.2f}x"
    check_index_structure(idx, wl.L, budget)
    # the selection is Algorithm 1 run on the scores the GPU itself produced: bit-exact, no tolerance
    assert idx.tolist() == oracle.allocate(scores, kernels, budget).tolist()
    rep = index_set_report(idx, want_scores, kernels, budget)
    assert not rep["unexcused"], rep
    return idx, scores, rep


def test_end_to_end_cfg1():
    _announce("end_to_end cfg1")
    inp = inputs.config(1)
    idx, scores, rep = _end_to_end(inp, inp.workload.pool_kernels, inp.workload.budget)
    mask = inp.needle_mask
    assert mask[idx].sum() >= 0.95 * mask.sum()


def test_end_to_end_cfg2():
    _announce("end_to_end cfg2")
    inp = inputs.config(2)
    idx, scores, rep = _end_to_end(inp, inp.workload.pool_kernels, inp.workload.budget)
    mask = inp.needle_mask
    assert mask[idx].sum() >= 0.95 * mask.sum()


def test_end_to_end_ragged_bf16():
    _announce("end_to_end ragged bf16")
    inp = inputs.custom(L=9001, Lq=40, Hq=16, Hkv=4, d=128, dtype="bf16", n_spans=3, span_len=(16, 40),
                        channel_scale=True, seed=77)
    _end_to_end(inp, (1, 3, 7, 15, 31), 512)


def _end_to_end_max_avg(inp, mk, ak, budget, sink):
    """Whole path with Algorithm 1 as printed: scores within tolerance of the oracle's, bit-identical to
    the window-max entry point's (same scoring kernels), indices equal to the staged call on those scores,
    and equal to the oracle's set up to tokens at a combination's threshold."""
    q, k = to_device(inp.q), to_device(inp.k)
    idx, count, scores = il.ilre_recall_max_avg(q, k, budget, mk, ak, sink)
    _, ref_scores = il.ilre_recall(q, k, min(budget, 64), (3,))
    staged_idx, staged_count = il.ilre_select_max_avg(scores, budget, mk, ak, sink)
    torch.cuda.synchronize()
    assert torch.equal(scores, ref_scores)
    assert torch.equal(idx, staged_idx) and int(count.item()) == int(staged_count.item())
    n = int(count.item())
    idx, scores = idx.cpu().numpy(), scores.cpu().numpy()
    want_scores, _, _ = oracle.scores(inp.q, inp.k)
    bad, worst = score_errors(scores, want_scores)
    assert bad == 0, f"{bad} scores out of tolerance, worst {worst:.2f}x"
    assert (idx[:sink] == np.arange(sink)).all() and (np.diff(idx[:n].astype(np.int64)) > 0).all()
    assert (idx[n:] == -1).all() and idx[:n].max() < inp.workload.L
    # Algorithm 1 as printed on the scores the GPU itself produced: bit-exact, no tolerance
    assert idx[:n].tolist() == oracle.allocate_max_avg(scores, mk, ak, budget, sink=sink).tolist()
    rep = index_set_report_max_avg(idx[:n], want_scores, mk, ak, budget, sink)
    assert not rep["unexcused"], rep
    return idx[:n], rep


def test_end_to_end_max_avg_cfg1():
    _announce("end_to_end max/avg cfg1 (paper default pooling set, sink 4)")
    inp = inputs.config(1)
    idx, rep = _end_to_end_max_avg(inp, PAPER_MAX, PAPER_AVG, inp.workload.budget, 4)
    mask = inp.needle_mask
    assert mask[idx].sum() >= 0.95 * mask.sum()


def test_end_to_end_max_avg_cfg2():
    _announce("end_to_end max/avg cfg2 (paper default pooling set, sink 4)")
    inp = inputs.config(2)
    idx, rep = _end_to_end_max_avg(inp, PAPER_MAX, PAPER_AVG, inp.workload.budget, 4)
    mask = inp.needle_mask
    assert mask[idx].sum() >= 0.95 * mask.sum()


def test_end_to_end_max_avg_ragged_bf16():
    _announce("end_to_end max/avg ragged bf16")
    inp = inputs.custom(L=9001, Lq=40, Hq=16, Hkv=4, d=128, dtype="bf16", n_spans=3, span_len=(16, 40),
                        channel_scale=True, seed=77)
    _end_to_end_max_avg(inp, (4,), (5,), 512, 0)          # the paper's One-Max-Avg ablation setting
    _end_to_end_max_avg(inp, PAPER_MAX, tuple(range(1, 10)), 1000, 4)   # Less-Avg-Kernels


def test_gather_ids_is_the_compressed_prompt():
    """Last line of Algorithm 1, C[I]: by definition the input IDs at the returned indices."""
    _announce("gather ids")
    rng = np.random.default_rng(17)
    # a normal selection, and one whose candidates run out (21 tokens, cells of 8: 16 reachable, budget 20)
    for L, budget, mk, ak, sink, short in ((50000, 3000, (2, 4, 8), (1, 2, 3), 4, False), (21, 20, (8,), (1,), 0, True)):
        ids = rng.integers(0, 128256, size=L).astype(np.int32)
        s = _scores_for("needles", L, rng) if L > 300 else rng.random(L).astype(np.float32)
        idx, count = il.ilre_select_max_avg(torch.from_numpy(s).cuda(), budget, mk, ak, sink)
        got = il.ilre_gather_ids(torch.from_numpy(ids).cuda(), idx)
        torch.cuda.synchronize()
        idx_h, n = idx.cpu().numpy(), int(count.item())
        assert (n < idx_h.size) == short and (idx_h[n:] == -1).all()
        want = np.where(idx_h >= 0, ids[np.clip(idx_h, 0, L - 1)], -1)
        assert got.cpu().numpy().tolist() == want.tolist()


def test_token_major_strides():
    _announce("token-major strided K and strided Q")
    inp = inputs.custom(L=2500, Lq=16, Hq=8, Hkv=2, d=128, dtype="bf16", n_spans=1, span_len=(16, 16), seed=5)
    q, k = to_device(inp.q), to_device(inp.k)
    k_tm = k.permute(1, 0, 2).contiguous().permute(1, 0, 2)          # storage [L, Hkv, d]
    q_pad = torch.zeros(8, 16, 256, dtype=q.dtype, device="cuda")[:, :, :128]
    q_pad.copy_(q)
    a_idx, a_sc = il.ilre_recall(q, k, 128, (3, 7))
    b_idx, b_sc = il.ilre_recall(q_pad, k_tm, 128, (3, 7))
    torch.cuda.synchronize()
    assert torch.equal(a_idx, b_idx) and torch.equal(a_sc, b_sc)


def test_bitwise_reproducible():
    _announce("run-to-run determinism")
    inp = inputs.custom(L=20000, Lq=64, Hq=8, Hkv=2, d=128, dtype="bf16", n_spans=4, span_len=(16, 64), seed=6)
    q, k = to_device(inp.q), to_device(inp.k)
    first = il.ilre_recall(q, k, 1024, (1, 3, 7, 15, 31))
    for _ in range(3):
        again = il.ilre_recall(q, k, 1024, (1, 3, 7, 15, 31))
        torch.cuda.synchronize()
        assert torch.equal(first[0], again[0]) and torch.equal(first[1], again[1])


def test_column_scores_do_not_depend_on_how_the_tokens_are_cut():
    """Long contexts: the second scoring pass sizes each workgroup's token range by how fast its XCD ran the first
    pass (a table the first pass leaves in the workspace).  The scores must be the same bits with that table, without
    it (a workspace nothing was left in), with a workspace full of noise, and inside the whole path."""
    _announce("second pass: token ranges from the XCDs' speed vs even ranges")
    L, Lq, Hq, Hkv = 1100000, 64, 8, 2   # 253 token ranges of 68 tiles (64 tokens each) per kv head
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    q = torch.randn(Hq, Lq, 128, device="cuda", generator=g).to(torch.bfloat16)
    k = torch.randn(Hkv, L, 128, device="cuda", generator=g).to(torch.bfloat16)
    nbytes = il.ilre_workspace_bytes(L, Lq, Hq, Hkv, 128, 5, il.ILRE_BF16)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    rmax, rsum = il.ilre_row_stats(q, k, workspace=ws)
    with_table = il.ilre_col_scores(q, k, rmax, rsum, workspace=ws).clone()
    clean = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    without = il.ilre_col_scores(q, k, rmax, rsum, workspace=clean).clone()
    noise = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=g)
    noisy = il.ilre_col_scores(q, k, rmax, rsum, workspace=noise).clone()
    idx, whole = il.ilre_recall(q, k, 2048, (1, 3, 7, 15, 31), workspace=ws)
    # a stand-alone selection uses the workspace from its base and may write over what the first pass left there
    il.ilre_row_stats(q, k, workspace=ws)
    il.ilre_select(whole, 2048, (1, 3, 7, 15, 31), workspace=ws)
    after_select = il.ilre_col_scores(q, k, rmax, rsum, workspace=ws).clone()
    torch.cuda.synchronize()
    assert torch.equal(with_table, without)
    assert torch.equal(with_table, noisy)
    assert torch.equal(with_table, whole)
    assert torch.equal(with_table, after_select)
    total = float(with_table.double().sum())
    assert abs(total - Hq * Lq) < 1e-3 * Hq * Lq  # every softmax row sums to one (Section 3.2, Eq. 4)


def test_custom_scale():
    _announce("custom softmax scale")
    inp = inputs.custom(L=1500, Lq=8, Hq=4, Hkv=2, d=128, dtype="bf16", seed=8)
    q, k = to_device(inp.q), to_device(inp.k)
    want, _, _ = oracle.scores(inp.q, inp.k, scale=0.05)
    _, got = il.ilre_recall(q, k, 64, (3,), scale=0.05)
    torch.cuda.synchronize()
    bad, worst = score_errors(got.cpu().numpy(), want)
    assert bad == 0, worst


@pytest.mark.parametrize("dtype,Lq", [("f32", 16), ("bf16", 64), ("bf16", 256)])
def test_extreme_logits_take_the_safe_row_statistics_path(dtype, Lq):
    """A key far above everything seen in the first tiles of its split: sums against a frozen
    reference leave the fp32 range, and the row statistics must come from the always-safe redo."""
    _announce(f"extreme logits {dtype} Lq={Lq}")
    L, Hq, Hkv = 6000, 4, 2
    inp = inputs.custom(L=L, Lq=Lq, Hq=Hq, Hkv=Hkv, d=128, dtype=dtype, seed=31)
    qf = inputs.as_float(inp.q).copy()
    kf = inputs.as_float(inp.k).copy()
    kf[0, 4500, :] = 12.0 * qf[0, 0, :]          # logit of row (0,0) ~ 12*128/sqrt(128) = 136 nats = 196 base-2 units
    kf[1, 5100, :] = -14.0 * qf[3, 1, :]
    if dtype == "bf16":
        q_in, k_in = inputs.f32_to_bf16_bits(qf), inputs.f32_to_bf16_bits(kf)
    else:
        q_in, k_in = qf, kf
    want_score, want_max, want_sum = oracle.scores(q_in, k_in)
    assert want_max.max() > 100.0
    q, k = to_device(q_in), to_device(k_in)
    row_max, row_sumexp = il.ilre_row_stats(q, k)
    scores = il.ilre_col_scores(q, k, row_max, row_sumexp)
    torch.cuda.synchronize()
    gm, gz = row_max.cpu().numpy().astype(np.float64), row_sumexp.cpu().numpy().astype(np.float64)
    assert np.isfinite(gm).all() and np.isfinite(gz).all()
    np.testing.assert_allclose(gm + np.log(gz), want_max + np.log(want_sum), rtol=2e-5, atol=2e-4)
    bad, worst = score_errors(scores.cpu().numpy(), want_score)
    assert bad == 0, f"{bad} scores out of tolerance, worst {worst:.2f}x"


def test_recall_replays_from_a_captured_graph():
    """The library neither allocates nor synchronises, so a whole recall step can be captured into a HIP
    graph; every replay, with eager work and synchronisations in between, gives the eager result."""
    _announce("graph capture and replay")
    inp = inputs.custom(L=30000, Lq=64, Hq=8, Hkv=2, d=128, dtype="bf16", n_spans=4, span_len=(16, 64), seed=12)
    q, k = to_device(inp.q), to_device(inp.k)
    kernels, budget, mk, ak = (1, 3, 7, 15, 31), 1024, (2, 4, 8), tuple(range(1, 17))
    ws = il.alloc_workspace(30000, 64, 8, 2, 128, len(kernels), il.ILRE_BF16)
    ws2 = il.alloc_workspace_max_avg(30000, 64, 8, 2, 128, 4, mk, len(ak), il.ILRE_BF16)
    eager_idx, eager_sc = il.ilre_recall(q, k, budget, kernels, workspace=ws)
    eager_pidx, eager_cnt, _ = il.ilre_recall_max_avg(q, k, budget, mk, ak, 4, workspace=ws2)
    torch.cuda.synchronize()
    eager_idx, eager_sc, eager_pidx = eager_idx.clone(), eager_sc.clone(), eager_pidx.clone()
    out_idx, out_sc = torch.empty_like(eager_idx), torch.empty_like(eager_sc)
    out_pidx, out_cnt, out_psc = torch.empty_like(eager_pidx), torch.empty_like(eager_cnt), torch.empty_like(eager_sc)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        il.ilre_recall(q, k, budget, kernels, workspace=ws, out_idx=out_idx, out_scores=out_sc)       # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            il.ilre_recall(q, k, budget, kernels, workspace=ws, out_idx=out_idx, out_scores=out_sc)
            il.ilre_recall_max_avg(q, k, budget, mk, ak, 4, workspace=ws2, out_idx=out_pidx, out_count=out_cnt,
                                   out_scores=out_psc)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        out_idx.fill_(-7)
        out_sc.zero_()
        out_pidx.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_idx, eager_idx) and torch.equal(out_sc, eager_sc), f"replay {rep}"
        assert torch.equal(out_pidx, eager_pidx) and int(out_cnt.item()) == int(eager_cnt.item()), f"replay {rep}"
        # eager work between the replays
        again, _ = il.ilre_recall(q, k, budget, kernels, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(again, eager_idx)


@pytest.mark.parametrize("seed", range(6))
def test_select_randomised_against_oracle(seed):
    """Many small random problems per seed, both forms of Algorithm 1: sizes around the chunk, bin and list
    boundaries of the kernels, score distributions with and without ties, all bit-exact with the oracle."""
    _announce(f"randomised selection, seed {seed}")
    rng = np.random.default_rng(9000 + seed)
    kinds = ("random", "few_values", "two_values", "equal", "narrow", "needles")
    for case in range(40):
        L = int(rng.choice([1, 2, 63, 64, 65, 255, 256, 257, 511, 513, 1000, 2047, 2049, 4097, 9999, 20000]))
        L = max(1, L + int(rng.integers(-3, 4)))
        kind = kinds[int(rng.integers(len(kinds)))]
        s = _scores_for(kind, L, rng) if L > 400 or kind != "needles" else rng.random(L).astype(np.float32)
        budget = int(rng.choice([1, 2, 7, 64, 255, 1000, 4096, 8192]))
        if min(budget, L) > 8192:
            budget = 8192
        dev = torch.from_numpy(s).cuda()
        if case % 2 == 0:
            n = int(rng.integers(1, 7))
            kernels = tuple(int(2 * rng.integers(0, 40) + 1) for _ in range(n))
            sink = int(rng.integers(0, min(L, 6) + 1)) if case % 4 == 0 else 0
            want = oracle.allocate(s, kernels, budget, sink=sink)
            got = il.ilre_select(dev, budget, kernels, sink=sink)
            torch.cuda.synchronize()
            assert got.cpu().numpy().tolist() == want.tolist(), (seed, case, L, kind, budget, kernels, sink)
        else:
            mk = tuple(int(rng.integers(1, 20)) for _ in range(int(rng.integers(1, 4))))
            ak = tuple(int(rng.integers(1, 24)) for _ in range(int(rng.integers(1, 5))))
            sink = int(rng.integers(0, min(L, 6) + 1))
            want = oracle.allocate_max_avg(s, mk, ak, budget, sink=sink)
            got, count = il.ilre_select_max_avg(dev, budget, mk, ak, sink)
            torch.cuda.synchronize()
            n_got = int(count.item())
            got = got.cpu().numpy()
            assert got[:n_got].tolist() == want.tolist() and (got[n_got:] == -1).all(), (seed, case, L, kind, budget, mk, ak, sink)
