"""Pins for the scoring oracle (Eq. 4 / Eq. 5): closed forms, invariants, a library softmax,
brute force on tiny inputs.  CPU only."""
import json
import math
import os

import numpy as np
import pytest
import scipy.special

import inputs
import oracle
from brute import brute_scores


def _rand(Hq, Hkv, Lq, L, d, seed, dtype=np.float32):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((Hq, Lq, d)).astype(dtype)
    k = rng.standard_normal((Hkv, L, d)).astype(dtype)
    return q, k


def test_golden_closed_forms(golden_dir):
    with open(os.path.join(golden_dir, "softmax_closed_form.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        q = np.array(c["q"], dtype=np.float32)
        k = np.log(np.array(c["k_log_of"], dtype=np.float64)).astype(np.float32)[:, :, None]
        score, _, _ = oracle.scores(q, k, scale=c["scale"])
        expect = np.array(c["expect_score_num"], dtype=np.float64) / c["expect_score_den"]
        # fp32 storage of ln(2), ln(3), ln(5) moves the probabilities by a few 1e-8
        np.testing.assert_allclose(score, expect, rtol=0, atol=2e-7, err_msg=c["name"])


def test_total_score_is_rows():
    # every softmax row sums to one, so the summed scores total Hq*Lq
    for (Hq, Hkv, Lq, L, d, seed) in [(4, 2, 3, 37, 8, 0), (8, 8, 5, 129, 16, 1), (6, 2, 1, 64, 4, 2)]:
        q, k = _rand(Hq, Hkv, Lq, L, d, seed)
        score, _, rsum = oracle.scores(q * 3, k)
        assert abs(score.sum() - Hq * Lq) < 1e-9 * Hq * Lq
        assert (rsum >= 1.0).all()


def test_equal_keys_give_uniform_score():
    q, k = _rand(4, 2, 3, 50, 8, 3)
    k[:] = k[:, :1, :]
    score, rmax, rsum = oracle.scores(q, k)
    np.testing.assert_allclose(score, 4 * 3 / 50, rtol=1e-12)
    np.testing.assert_allclose(rsum, 50.0, rtol=1e-12)
    score0, _, _ = oracle.scores(np.zeros_like(q), _rand(4, 2, 3, 50, 8, 4)[1])
    np.testing.assert_allclose(score0, 4 * 3 / 50, rtol=1e-12)


def test_dominant_key_takes_all_mass():
    Hq, Hkv, Lq, L, d = 4, 2, 3, 40, 8
    rng = np.random.default_rng(5)
    direction = rng.standard_normal(d).astype(np.float32)
    q = np.tile(direction, (Hq, Lq, 1)).astype(np.float32)
    k = (0.01 * rng.standard_normal((Hkv, L, d))).astype(np.float32)
    k[:, 17, :] = 200.0 * direction
    score, _, _ = oracle.scores(q, k)
    assert abs(score[17] - Hq * Lq) < 1e-9
    assert score[np.arange(L) != 17].max() < 1e-12


def test_matches_library_softmax_with_gqa_repeat():
    for dtype, seed in [(np.float32, 6), ("bf16", 7)]:
        Hq, Hkv, Lq, L, d = 8, 2, 5, 203, 16
        q, k = _rand(Hq, Hkv, Lq, L, d, seed)
        if dtype == "bf16":
            qb, kb = inputs.f32_to_bf16_bits(q), inputs.f32_to_bf16_bits(k)
            q, k = inputs.bf16_bits_to_f32(qb), inputs.bf16_bits_to_f32(kb)
            score, rmax, rsum = oracle.scores(qb, kb)
        else:
            score, rmax, rsum = oracle.scores(q, k)
        krep = np.repeat(k.astype(np.float64), Hq // Hkv, axis=0)           # kv head g serves heads g*G..g*G+G-1
        logits = np.einsum("hid,htd->hit", q.astype(np.float64), krep) / math.sqrt(d)
        p = scipy.special.softmax(logits, axis=-1)
        np.testing.assert_allclose(score, p.sum(axis=(0, 1)), rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(rmax, logits.max(-1).ravel(), rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(rsum, np.exp(logits - logits.max(-1, keepdims=True)).sum(-1).ravel(), rtol=1e-12)
        smax, _, _ = oracle.scores(qb, kb, mode=oracle.MODE_MAX) if dtype == "bf16" else oracle.scores(q, k, mode=oracle.MODE_MAX)
        np.testing.assert_allclose(smax, p.max(axis=(0, 1)), rtol=1e-12, atol=1e-15)


def test_gqa_mapping_is_consecutive():
    # kv head 0 carries a needle at token 3, kv head 1 at token 9.  Query heads 0,1 -> kv 0 and
    # heads 2,3 -> kv 1 under consecutive grouping; only head 0 looks along the needle direction.
    Hq, Hkv, Lq, L, d = 4, 2, 1, 12, 4
    q = np.zeros((Hq, Lq, d), dtype=np.float32)
    k = np.zeros((Hkv, L, d), dtype=np.float32)
    q[0, 0, 0] = 50.0
    k[0, 3, 0] = 1.0
    k[1, 9, 0] = 1.0
    score, _, _ = oracle.scores(q, k, scale=1.0)
    assert score[3] > 1.0 and score[9] < 0.5          # interleaved mapping would not change this...
    q[:] = 0
    q[1, 0, 0] = 50.0                                 # ...but head 1 tells the two mappings apart:
    score, _, _ = oracle.scores(q, k, scale=1.0)      # consecutive -> kv 0 (token 3); interleaved -> kv 1 (token 9)
    assert score[3] > 1.0 and score[9] < 0.5
    q[:] = 0
    q[2, 0, 0] = 50.0
    score, _, _ = oracle.scores(q, k, scale=1.0)
    assert score[9] > 1.0 and score[3] < 0.5


def test_gqa_equals_mha_with_repeated_kv():
    q, k = _rand(8, 2, 3, 41, 8, 8)
    a, _, _ = oracle.scores(q, k)
    b, _, _ = oracle.scores(q, np.repeat(k, 4, axis=0))
    np.testing.assert_allclose(a, b, rtol=1e-13)


def test_permutation_equivariance():
    q, k = _rand(4, 2, 3, 33, 8, 9)
    rng = np.random.default_rng(10)
    base, _, _ = oracle.scores(q, k)
    perm = rng.permutation(33)
    moved, _, _ = oracle.scores(q, k[:, perm, :])
    np.testing.assert_allclose(moved, base[perm], rtol=1e-12)
    qperm = q[:, rng.permutation(3), :]
    same, _, _ = oracle.scores(qperm, k)
    np.testing.assert_allclose(same, base, rtol=1e-12)
    qswap = q[[1, 0, 3, 2]]                           # swap heads inside each group
    same2, _, _ = oracle.scores(qswap, k)
    np.testing.assert_allclose(same2, base, rtol=1e-12)


@pytest.mark.parametrize("mode", ["sum", "max"])
def test_brute_force_tiny(mode):
    Hq, Hkv, Lq, L, d = 4, 2, 3, 37, 8
    q, k = _rand(Hq, Hkv, Lq, L, d, 11)
    scale = 1.0 / math.sqrt(d)
    want = brute_scores(q.astype(float).tolist(), k.astype(float).tolist(), Hq, Hkv, Lq, L, d, scale, mode)
    got, _, _ = oracle.scores(q, k, mode=oracle.MODE_SUM if mode == "sum" else oracle.MODE_MAX)
    np.testing.assert_allclose(got, want, rtol=1e-12)


def test_row_stats_subset_matches_full():
    q, k = _rand(4, 2, 5, 70, 8, 12)
    _, rmax, rsum = oracle.scores(q, k)
    rows = [0, 7, 13, 19]
    m, z = oracle.row_stats(q, k, rows)
    np.testing.assert_allclose(m, rmax[rows], rtol=0, atol=0)
    np.testing.assert_allclose(z, rsum[rows], rtol=1e-15)


def test_single_token_context():
    q, k = _rand(4, 2, 3, 1, 8, 13)
    score, _, rsum = oracle.scores(q, k)
    assert score.shape == (1,) and abs(score[0] - 12) < 1e-12 and (rsum == 1.0).all()
