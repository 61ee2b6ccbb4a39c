"""Pins for the allocation oracle (Algorithm 1, stride-1 max-pool reading).  CPU only."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from brute import brute_allocate, brute_pool


def test_golden_worked_examples(golden_dir):
    with open(os.path.join(golden_dir, "allocation_worked.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        got = oracle.allocate(np.array(c["score"], dtype=np.float32), c["kernels"], c["budget"])
        assert got.tolist() == c["expect"], c["name"]


def test_kernel_one_is_identity_and_plain_topk():
    rng = np.random.default_rng(0)
    s = rng.random(500).astype(np.float32)
    assert (oracle.max_pool_same(s, 1) == s).all()
    got = oracle.allocate(s, [1], 40)
    want = np.sort(np.argsort(-s, kind="stable")[:40])
    assert got.tolist() == want.tolist()


@pytest.mark.parametrize("w", [1, 3, 7, 15, 31, 63])
@pytest.mark.parametrize("L", [1, 2, 5, 31, 200])
def test_pool_matches_library_and_brute(w, L):
    rng = np.random.default_rng(w * 1000 + L)
    s = rng.random(L).astype(np.float32)
    got = oracle.max_pool_same(s, w)
    assert got.tolist() == brute_pool(s.tolist(), w)
    if (w - 1) // 2 <= L // 2 or True:
        pad = (w - 1) // 2
        x = torch.from_numpy(s)[None, None, :]
        x = torch.nn.functional.pad(x, (pad, pad), value=float("-inf"))
        lib = torch.nn.functional.max_pool1d(x, kernel_size=w, stride=1)[0, 0].numpy()
        assert got.tolist() == lib.tolist()


def test_even_kernel_rejected():
    with pytest.raises(ValueError):
        oracle.max_pool_same(np.ones(4, dtype=np.float32), 2)


def test_split_budget():
    assert oracle.split_budget(256, 3) == [86, 85, 85]
    assert oracle.split_budget(4096, 5) == [820, 819, 819, 819, 819]
    assert oracle.split_budget(4096, 4) == [1024] * 4
    for b in range(1, 40):
        for n in range(1, 9):
            sh = oracle.split_budget(b, n)
            assert sum(sh) == b and max(sh) - min(sh) <= 1 and sh == sorted(sh, reverse=True)


def test_all_equal_scores_take_lowest_indices():
    s = np.full(100, 0.25, dtype=np.float32)
    assert oracle.allocate(s, [3, 7, 15], 10).tolist() == list(range(10))


def test_structure_invariants():
    rng = np.random.default_rng(1)
    for L, B, kernels in [(300, 64, [3, 7, 15]), (50, 80, [1, 3]), (17, 17, [31]), (9, 4, [3, 3, 3, 3, 3, 3])]:
        s = rng.random(L).astype(np.float32)
        idx = oracle.allocate(s, kernels, B)
        assert len(idx) == min(B, L)
        assert (np.diff(idx) > 0).all()
        assert idx.min() >= 0 and idx.max() < L


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_allocation(seed):
    rng = np.random.default_rng(100 + seed)
    L = int(rng.integers(5, 64))
    # few distinct values -> many exact ties, as stride-1 pooling produces on real scores
    s = (rng.integers(0, 6, size=L) / 8.0 + 0.125).astype(np.float32)
    kernels = [int(x) for x in rng.choice([1, 3, 5, 7, 9], size=int(rng.integers(1, 4)))]
    B = int(rng.integers(1, L + 5))
    assert oracle.allocate(s, kernels, B).tolist() == brute_allocate(s.tolist(), kernels, B)


def test_order_of_kernels_matters_through_allocated_set():
    s = np.array([0.1, 0.9, 0.2, 0.3, 0.8, 0.05, 0.6, 0.7, 0.15, 0.25], dtype=np.float32)
    a = oracle.allocate(s, [1, 3], 4).tolist()
    b = oracle.allocate(s, [3, 1], 4).tolist()
    assert a == [0, 1, 2, 4] and b == [0, 1, 4, 7] and a != b


def test_thresholds_replay():
    rng = np.random.default_rng(2)
    s = rng.random(400).astype(np.float32)
    th = oracle.thresholds(s, [3, 7], 20)
    idx = oracle.allocate(s, [3, 7], 20)
    pooled3, thr3 = th[0]
    assert (pooled3 == oracle.max_pool_same(s, 3)).all()
    # every token strictly above a kernel's threshold in its pooled vector is allocated by then
    assert set(np.flatnonzero(pooled3 > thr3)).issubset(set(idx.tolist()))


# ---- Algorithm 1 as printed: strided max pooling then average pooling ---------------------------

from brute import brute_allocate_max_avg  # noqa: E402


def test_golden_max_avg_examples(golden_dir):
    with open(os.path.join(golden_dir, "allocation_worked.json")) as f:
        cases = json.load(f)["max_avg_cases"]
    for c in cases:
        got = oracle.allocate_max_avg(np.array(c["score"], dtype=np.float32), c["max_kernels"], c["avg_kernels"],
                                      c["budget"], sink=c["sink"])
        assert got.tolist() == c["expect"], c["name"]


@pytest.mark.parametrize("m", [1, 2, 4, 8])
def test_strided_max_matches_library(m):
    rng = np.random.default_rng(m)
    s = rng.random(203).astype(np.float32)
    lib = torch.nn.functional.max_pool1d(torch.from_numpy(s)[None, None, :], kernel_size=m, stride=m)[0, 0].numpy()
    assert oracle.max_pool_strided(s, m).tolist() == lib.tolist()


@pytest.mark.parametrize("n", list(range(1, 17)))
def test_avg_pool_matches_library_up_to_rounding_and_index_shift(n):
    rng = np.random.default_rng(100 + n)
    x = rng.random(77).astype(np.float32)
    got = oracle.avg_pool_same(x, n)
    # torch pads n//2 zeros on both sides and counts them: its output q averages [q - n//2, q + (n-1)//2 ... ],
    # i.e. for even n the same windows shifted by one cell
    lib = torch.nn.functional.avg_pool1d(torch.from_numpy(x)[None, None, :], kernel_size=n, stride=1, padding=n // 2,
                                         count_include_pad=True)[0, 0].numpy()
    lib = lib[1:] if n % 2 == 0 else lib
    np.testing.assert_allclose(got, lib[:77], rtol=2e-6, atol=1e-7)
    # and exactly the float32 left-to-right definition
    for p in (0, 1, 38, 76):
        acc = np.float32(0)
        for q in range(p - (n - 1) // 2, p + n // 2 + 1):
            acc = np.float32(acc + (x[q] if 0 <= q < 77 else np.float32(0)))
        assert got[p] == np.float32(acc / np.float32(n))


def test_kernel_one_max_and_avg_is_plain_topk_with_cap():
    rng = np.random.default_rng(3)
    s = rng.random(300).astype(np.float32)
    got = oracle.allocate_max_avg(s, [1], [1], 40)
    want = np.sort(np.argsort(-s, kind="stable")[:40])
    assert got.tolist() == want.tolist()


@pytest.mark.parametrize("seed", range(8))
def test_brute_force_max_avg(seed):
    rng = np.random.default_rng(200 + seed)
    L = int(rng.integers(9, 90))
    s = (rng.integers(0, 12, size=L) / 16.0 + 0.0625).astype(np.float32) if seed % 2 else rng.random(L).astype(np.float32)
    mk = [int(x) for x in rng.choice([1, 2, 4, 8], size=int(rng.integers(1, 4)), replace=False)]
    ak = [int(x) for x in rng.choice(np.arange(1, 9), size=int(rng.integers(1, 4)), replace=False)]
    B = int(rng.integers(1, L + 3))
    sink = int(rng.integers(0, 4))
    assert oracle.allocate_max_avg(s, mk, ak, B, sink=sink).tolist() == brute_allocate_max_avg(s.tolist(), mk, ak, B, sink)


def test_max_avg_structure():
    rng = np.random.default_rng(9)
    s = rng.random(5000).astype(np.float32)
    idx = oracle.allocate_max_avg(s, [2, 4, 8], list(range(1, 17)), 480, sink=4)
    assert idx[:4].tolist() == [0, 1, 2, 3] and (np.diff(idx) > 0).all() and len(idx) <= 4 + 480 and idx.max() < 5000


def test_thresholds_max_avg_replay():
    """The replay used by the index-set comparison rule agrees with allocate_max_avg: every admitted token's
    value in some combination is at or above what that combination last admitted, and nothing below a
    combination's cap value was ever a candidate of it."""
    rng = np.random.default_rng(5)
    s = rng.random(4000).astype(np.float32)
    mk, ak, B, sink = [2, 4, 8], [1, 2, 3, 8], 600, 4
    idx = oracle.allocate_max_avg(s, mk, ak, B, sink=sink)
    th = oracle.thresholds_max_avg(s, mk, ak, B, sink=sink)
    assert len(th) == len(mk) * len(ak)
    for per_token, last, cap in th:
        assert per_token.shape == (4000,) and np.isnan(per_token[:sink]).all()
        assert last is not None and cap is not None and last >= cap
    body = idx[idx >= sink]
    admitted_somewhere = np.zeros(len(body), dtype=bool)
    for per_token, last, cap in th:
        admitted_somewhere |= per_token[body] >= last
    assert admitted_somewhere.all()
    # m = 4: tokens after the last whole cell have no value in that combination
    th2 = oracle.thresholds_max_avg(s[:1003], [4], [1], 50, sink=0)
    assert np.isnan(th2[0][0][1000:]).all() and not np.isnan(th2[0][0][:1000]).any()
    assert th2[0][2] == float(np.sort(s[:1000].reshape(250, 4).max(axis=1))[::-1][50 // 4])


def test_allocate_with_a_sink_part_against_brute_force():
    """The sink tokens are always kept, the pooling windows stop at the sink boundary (a high sink score must not
    leak into its neighbours' pooled values) and the budget counts the other tokens."""
    rng = np.random.default_rng(41)
    for case in range(30):
        L = int(rng.integers(5, 60))
        sink = int(rng.integers(0, min(L, 6) + 1))
        s = (rng.integers(1, 12, size=L) / 16.0).astype(np.float32) if case % 2 else rng.random(L).astype(np.float32)
        s[:sink] = 50.0                                   # would win every window it leaked into
        kernels = [int(2 * rng.integers(0, 5) + 1) for _ in range(int(rng.integers(1, 4)))]
        budget = int(rng.integers(1, L + 3))
        got = oracle.allocate(s, kernels, budget, sink=sink)
        assert got.tolist() == brute_allocate([float(x) for x in s], kernels, budget, sink=sink)
        assert got[:sink].tolist() == list(range(sink)) and len(got) == sink + min(budget, L - sink)
    # hand-worked: scores 9 9 | 1 5 1 1 4 1, sink 2, kernel 3, budget 3 -> body pooled 5 5 5 4 4 4 -> body tokens 0 1 2
    s = np.array([9, 9, 1, 5, 1, 1, 4, 1], dtype=np.float32)
    assert oracle.allocate(s, [3], 3, sink=2).tolist() == [0, 1, 2, 3, 4]
