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
