"""Pins of the re-RoPE oracle (Section 3.3, second DCA equation) against things other than itself:
hand-worked values, complex-number rotation, the relative-position property of rotary embeddings,
invariants."""
import json
import os

import numpy as np
import pytest

import oracle


def _complex_rope(x, pos, inv_freq, pairing):
    """Independent route: a pair is a complex number, a rotation by `pos` positions multiplies it by
    exp(i * pos * inv_freq)."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    z = x[..., :d // 2] + 1j * x[..., d // 2:] if pairing == oracle.PAIR_HALF else x[..., 0::2] + 1j * x[..., 1::2]
    z = z * np.exp(1j * np.float64(pos) * inv_freq)
    out = np.empty_like(x)
    if pairing == oracle.PAIR_HALF:
        out[..., :d // 2], out[..., d // 2:] = z.real, z.imag
    else:
        out[..., 0::2], out[..., 1::2] = z.real, z.imag
    return out


def test_worked_example(golden_dir):
    with open(os.path.join(golden_dir, "rerope_worked.json")) as f:
        g = json.load(f)
    freq = oracle.default_inv_freq(4, g["base"])
    np.testing.assert_allclose(freq, [1.0, 0.01], rtol=1e-15)
    x = np.array(g["x"])
    np.testing.assert_allclose(oracle.rotate(x, g["distance"], freq, oracle.PAIR_HALF), g["half_split"], atol=2e-9)
    np.testing.assert_allclose(oracle.rotate(x, g["distance"], freq, oracle.PAIR_INTERLEAVED), g["interleaved"], atol=2e-9)
    c = g["chunks"]
    bounds = oracle.chunk_bounds(c["L"], c["chunk"], c["first_extra"])
    assert [list(b) for b in bounds] == c["bounds"]
    assert oracle.chunk_distances(len(bounds), c["chunk"]) == c["distances"]


@pytest.mark.parametrize("pairing", [oracle.PAIR_HALF, oracle.PAIR_INTERLEAVED])
def test_rotation_is_complex_multiplication(pairing):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 7, 128))
    freq = oracle.default_inv_freq(128, 500000.0)
    for dist in (0, 1, 1024, 999424):
        np.testing.assert_allclose(oracle.rotate(x, dist, freq, pairing), _complex_rope(x, dist, freq, pairing),
                                   rtol=0, atol=1e-9)


def test_rotation_invariants():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((3, 128))
    freq = oracle.default_inv_freq(128)
    y = oracle.rotate(x, 4096, freq)
    # pair norms are kept, distances add up, distance 0 is the identity
    np.testing.assert_allclose(y[:, :64] ** 2 + y[:, 64:] ** 2, x[:, :64] ** 2 + x[:, 64:] ** 2, rtol=1e-12)
    np.testing.assert_allclose(oracle.rotate(oracle.rotate(x, 1000, freq), 3096, freq), y, atol=1e-9)
    assert np.array_equal(oracle.rotate(x, 0, freq), x)
    # a wrong sign would rotate backwards
    assert not np.allclose(oracle.rotate(x, -4096, freq), y)


@pytest.mark.parametrize("pairing", [oracle.PAIR_HALF, oracle.PAIR_INTERLEAVED])
@pytest.mark.parametrize("L,chunk,extra", [(100, 16, 4), (64, 16, 0), (37, 50, 4), (33, 8, 1)])
def test_rerope_moves_every_chunk_to_the_base_chunk(L, chunk, extra, pairing):
    """The property the method wants: after the re-RoPE a key of chunk i scores against a query exactly as
    if it had been embedded D_i positions later, i.e. inside the base chunk; the last two chunks are untouched."""
    rng = np.random.default_rng(L)
    d, Hkv = 16, 2
    freq = oracle.default_inv_freq(d, 10000.0)
    raw = rng.standard_normal((Hkv, L, d))                                    # keys before any position embedding
    pos = np.arange(L)
    k = np.stack([_complex_rope(raw[:, t, :], pos[t], freq, pairing) for t in range(L)], axis=1)
    got = oracle.rerope_keys(k.astype(np.float32), chunk, extra, 10000.0, pairing=pairing)
    bounds = oracle.chunk_bounds(L, chunk, extra)
    n = len(bounds)
    q = _complex_rope(rng.standard_normal(d), L + 5, freq, pairing)           # a query embedded after the context
    for c, (start, end) in enumerate(bounds):
        shift = (n - 2 - c) * chunk if c < n - 2 else 0
        for t in range(start, end):
            moved = _complex_rope(raw[:, t, :], t + shift, freq, pairing)
            np.testing.assert_allclose(got[:, t, :] @ q, moved @ q, atol=1e-5)
            if shift == 0:
                assert np.array_equal(got[:, t, :], k.astype(np.float32)[:, t, :].astype(np.float64))
    # every key now sits within two chunk sizes (plus the first chunk's extra tokens) of the end of the context
    for c, (start, end) in enumerate(bounds):
        shift = (n - 2 - c) * chunk if c < n - 2 else 0
        assert L - (start + shift) <= 2 * chunk + extra


def test_bf16_bit_patterns_and_custom_frequencies():
    rng = np.random.default_rng(6)
    k32 = rng.standard_normal((1, 40, 8)).astype(np.float32)
    bits = (k32.view(np.uint32) >> 16).astype(np.uint16)                     # truncation is fine here: exact bf16 values
    exact = (bits.astype(np.uint32) << 16).view(np.float32)
    freq = np.array([0.5, 0.25, 0.125, 0.0625])
    a = oracle.rerope_keys(bits, 8, 0, inv_freq=freq)
    b = oracle.rerope_keys(exact, 8, 0, inv_freq=freq)
    assert np.array_equal(a, b)
    np.testing.assert_allclose(a[0, 0], _complex_rope(exact[0, 0], 3 * 8, freq, oracle.PAIR_HALF), atol=1e-12)


@pytest.mark.parametrize("pairing", [oracle.PAIR_HALF, oracle.PAIR_INTERLEAVED])
def test_turning_the_key_equals_turning_the_query_back(pairing):
    """R(D) is orthogonal: q . (R(D) k) = (R(-D) q) . k.  Pins the direction of the rotation of every
    chunk of `rerope_keys` from the other operand's side."""
    rng = np.random.default_rng(11)
    L, chunk, extra, d = 97, 16, 4, 16
    q = rng.standard_normal((3, d))
    k = rng.standard_normal((2, L, d)).astype(np.float32)
    freq = oracle.default_inv_freq(d, 100.0)
    kr = oracle.rerope_keys(k, chunk, extra, base=100.0, pairing=pairing)
    bounds = oracle.chunk_bounds(L, chunk, extra)
    turned = 0
    for (s0, e0), dist in zip(bounds, oracle.chunk_distances(len(bounds), chunk)):
        qc = oracle.rotate(q, -dist, freq, pairing)
        want = np.einsum("id,htd->hit", qc, k[:, s0:e0].astype(np.float64))
        got = np.einsum("id,htd->hit", q, kr[:, s0:e0])
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
        if dist:
            plain = np.einsum("id,htd->hit", q, k[:, s0:e0].astype(np.float64))
            turned += int(np.abs(got - plain).max() > 0.1)
    assert turned >= 3
