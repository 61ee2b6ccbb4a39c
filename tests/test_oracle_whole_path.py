"""Whole-path pins: brute force on tiny shapes, planted needles are recalled, and several
kernel sizes recall a long uneven span better than one (the paper's Section 3.2 observation
about long keys, checked qualitatively on synthetic scores).  CPU only."""
import math

import numpy as np

import inputs
import oracle
from brute import brute_allocate, brute_scores


def test_whole_path_brute_force():
    inp = inputs.custom(L=37, Lq=3, Hq=4, Hkv=2, d=8, dtype="f32", pool_kernels=(1, 3, 5), budget=7, seed=3)
    idx, score = oracle.recall(inp.q, inp.k, (1, 3, 5), 7)
    bs = brute_scores(inp.q.astype(float).tolist(), inp.k.astype(float).tolist(), 4, 2, 3, 37, 8, 1 / math.sqrt(8))
    np.testing.assert_allclose(score, bs, rtol=1e-12)
    b32 = [float(np.float32(x)) for x in bs]
    assert idx.tolist() == brute_allocate(b32, (1, 3, 5), 7)


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
