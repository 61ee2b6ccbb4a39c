"""Whole-path pins: brute force on tiny shapes, planted needles are recalled, and several
kernel sizes recall a long uneven span better than one (the paper's Section 3.2 observation
about long keys, checked qualitatively on synthetic scores).  CPU only."""
import math

import numpy as np

import inputs
import oracle
from brute import brute_allocate, brute_allocate_max_avg, brute_scores


def test_whole_path_brute_force():
    inp = inputs.custom(L=37, Lq=3, Hq=4, Hkv=2, d=8, dtype="f32", pool_kernels=(1, 3, 5), budget=7, seed=3)
    idx, score = oracle.recall(inp.q, inp.k, (1, 3, 5), 7)
    bs = brute_scores(inp.q.astype(float).tolist(), inp.k.astype(float).tolist(), 4, 2, 3, 37, 8, 1 / math.sqrt(8))
    np.testing.assert_allclose(score, bs, rtol=1e-12)
    b32 = [float(np.float32(x)) for x in bs]
    assert idx.tolist() == brute_allocate(b32, (1, 3, 5), 7)


def test_whole_path_as_printed_brute_force():
    """recall_max_avg (Eq. 4 over all positions, Eq. 5, then Algorithm 1 as printed with a sink part) against
    pure-Python loops: sum and max reduction, a sink that is not a multiple of any max kernel, a budget that
    the K_m cap and the shares do not divide."""
    for seed, (L, sink, mk, ak, budget), mode in ((4, (41, 3, (2, 4), (1, 2, 3), 11), "sum"),
                                                   (5, (29, 1, (3,), (2, 5), 9), "max"),
                                                   (6, (23, 4, (2, 8), (1, 4), 30), "sum")):
        inp = inputs.custom(L=L, Lq=2, Hq=4, Hkv=2, d=8, dtype="f32", seed=seed)
        omode = oracle.MODE_SUM if mode == "sum" else oracle.MODE_MAX
        idx, score = oracle.recall_max_avg(inp.q, inp.k, mk, ak, budget, sink=sink, mode=omode)
        bs = brute_scores(inp.q.astype(float).tolist(), inp.k.astype(float).tolist(), 4, 2, 2, L, 8, 1 / math.sqrt(8),
                          mode=mode)
        np.testing.assert_allclose(score, bs, rtol=1e-12)
        b32 = [float(np.float32(x)) for x in bs]
        want = brute_allocate_max_avg(b32, mk, ak, budget, sink=sink)
        assert idx.tolist() == want
        assert idx[:sink].tolist() == list(range(sink))            # the sink part is always kept
        # a plausible slip -- pooling the whole score vector instead of score[sink:] -- gives another set
        if seed == 4:
            shifted = oracle.allocate_max_avg(np.asarray(b32, dtype=np.float32), mk, ak, budget, sink=0)
            assert sorted(set(range(sink)) | set(shifted.tolist())) != want


def test_planted_needles_recalled_cfg1():
    inp = inputs.config(1)
    wl = inp.workload
    idx, score = oracle.recall(inp.q, inp.k, wl.pool_kernels, wl.budget)
    mask = inp.needle_mask
    assert abs(score.sum() - wl.Hq * wl.Lq) < 1e-6
    assert mask[idx].sum() >= 0.95 * mask.sum()
    assert len(idx) == wl.budget and (np.diff(idx) > 0).all()


def test_planted_needles_recalled_bf16_small():
    inp = inputs.custom(L=6000, Lq=16, Hq=8, Hkv=2, d=128, dtype="bf16", pool_kernels=(3, 7, 15, 31),
                        budget=256, n_spans=3, span_len=(32, 48), channel_scale=True, seed=21)
    idx, score = oracle.recall(inp.q, inp.k, (3, 7, 15, 31), 256)
    mask = inp.needle_mask
    assert abs(score.sum() - 8 * 16) < 1e-6
    assert mask[idx].sum() >= 0.95 * mask.sum()


def test_multi_kernel_recalls_long_uneven_span_better():
    # background noise, one 48-token span where only every 6th token scores high
    rng = np.random.default_rng(5)
    L, start, n = 4000, 1500, 48
    s = (0.01 + 0.01 * rng.random(L)).astype(np.float32)
    s[start:start + n:6] = 1.0
    budget = 48
    span = np.zeros(L, dtype=bool)
    span[start:start + n] = True
    single = oracle.allocate(s, [1], budget)
    multi = oracle.allocate(s, [1, 3, 7, 15, 31], budget)
    assert span[multi].sum() > span[single].sum() + 20
