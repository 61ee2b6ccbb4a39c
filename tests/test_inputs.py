"""The seeded generator: determinism, shapes, bf16 rounding, span placement.  CPU only."""
import numpy as np
import torch

import inputs


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(10000) * 10 ** rng.uniform(-6, 6, 10000)).astype(np.float32)
    bits = inputs.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (bits == ref).all()
    back = inputs.bf16_bits_to_f32(bits)
    assert (torch.from_numpy(back).to(torch.bfloat16).float().numpy() == back).all()


def test_deterministic_and_shaped():
    a = inputs.custom(L=300, Lq=4, Hq=8, Hkv=2, d=16, dtype="bf16", n_spans=2, span_len=(8, 12), seed=4)
    b = inputs.custom(L=300, Lq=4, Hq=8, Hkv=2, d=16, dtype="bf16", n_spans=2, span_len=(8, 12), seed=4)
    assert (a.q == b.q).all() and (a.k == b.k).all() and a.spans == b.spans
    assert a.q.shape == (8, 4, 16) and a.k.shape == (2, 300, 16) and a.q.dtype == np.uint16
    c = inputs.custom(L=300, Lq=4, Hq=8, Hkv=2, d=16, dtype="f32", seed=5)
    assert c.q.dtype == np.float32 and not c.spans


def test_spans_do_not_overlap_and_fit():
    rng = np.random.default_rng(1)
    spans = inputs.place_spans(rng, 5000, 20, 64, 128)
    taken = np.zeros(5000, dtype=int)
    for s, n in spans:
        assert 0 <= s and s + n <= 5000 and 64 <= n <= 128
        taken[s:s + n] += 1
    assert taken.max() == 1


def test_config_table_matches_targets():
    wl = inputs.CONFIGS[5]
    assert (wl.L, wl.Lq, wl.Hq, wl.Hkv, wl.d, wl.dtype) == (1048576, 256, 32, 8, 128, "bf16")
    assert wl.pool_kernels == (1, 3, 7, 15, 31) and wl.budget == 4096
    wl = inputs.CONFIGS[1]
    assert (wl.L, wl.Lq, wl.dtype, wl.pool_kernels, wl.budget) == (4096, 32, "f32", (3, 7, 15), 256)
