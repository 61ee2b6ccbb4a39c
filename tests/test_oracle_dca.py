"""Pins of the query-side DCA oracle (Section 3.3, second DCA equation, applied to the query instead of
the key) against things other than itself: the key-side re-RoPE oracle, the relative-position property
of rotary embeddings, the plain scoring oracle where no chunk is turned, a library bf16 conversion."""
import numpy as np
import pytest
import torch

import oracle


def _softmax_sum(logits):
    s = logits - logits.max(axis=2, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=2, keepdims=True)
    return p.sum(axis=(0, 1))


def _complex_rope(x, pos, inv_freq):
    d = x.shape[-1]
    z = (x[..., :d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * np.float64(pos) * inv_freq)
    return np.concatenate([z.real, z.imag], axis=-1)


@pytest.mark.parametrize("pairing", [oracle.PAIR_HALF, oracle.PAIR_INTERLEAVED])
@pytest.mark.parametrize("L,chunk,first_extra", [(97, 16, 4), (64, 16, 0), (50, 7, 3)])
def test_query_side_equals_key_side(pairing, L, chunk, first_extra):
    """Unrounded (fp32 inputs), turning the query by -D_i gives the logits of the turned cache."""
    rng = np.random.default_rng(11)
    Hq, Hkv, Lq, d = 4, 2, 3, 16
    q = rng.standard_normal((Hq, Lq, d)).astype(np.float32)
    k = rng.standard_normal((Hkv, L, d)).astype(np.float32)
    kr = oracle.rerope_keys(k, chunk, first_extra, base=100.0, pairing=pairing)  # fp64, key side
    want = np.einsum("hid,htd->hit", q.astype(np.float64), np.repeat(kr, Hq // Hkv, axis=0)) / np.sqrt(d)
    got = oracle.logits_dca(q, k, chunk, first_extra, base=100.0, pairing=pairing)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.scores_dca(q, k, chunk, first_extra, base=100.0, pairing=pairing),
                               _softmax_sum(want), rtol=1e-12)
    # the turn matters here: the plain logits are somewhere else
    plain = np.einsum("hid,htd->hit", q.astype(np.float64), np.repeat(k.astype(np.float64), Hq // Hkv, axis=0)) / np.sqrt(d)
    assert np.abs(got - plain).max() > 0.1


def test_relative_position_property():
    """Keys embedded at their positions, the query at position p_q: the logit of a token of chunk i is
    that of the un-embedded vectors at relative position p_t + D_i - p_q."""
    rng = np.random.default_rng(12)
    d, L, chunk, fe = 8, 45, 8, 2
    freq = oracle.default_inv_freq(d, 50.0)
    q0 = rng.standard_normal(d)
    k0 = rng.standard_normal((L, d))
    pq = L + 3
    k = np.stack([_complex_rope(k0[t], t, freq) for t in range(L)])[None].astype(np.float32)
    q = _complex_rope(q0, pq, freq)[None, None].astype(np.float32)
    got = oracle.logits_dca(q, k, chunk, fe, inv_freq=freq, scale=1.0)[0, 0]
    bounds = oracle.chunk_bounds(L, chunk, fe)
    dist = oracle.chunk_distances(len(bounds), chunk)
    assert len(bounds) == 6 and dist == [32, 24, 16, 8, 0, 0]
    for (s, e), D in zip(bounds, dist):
        for t in range(s, e):
            want = q0 @ _complex_rope(k0[t], t + D - pq, freq)
            assert abs(got[t] - want) < 2e-5  # the fp32 rounding of the embedded inputs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_no_turned_chunk_is_the_plain_score(dtype):
    """With one or two chunks nothing is turned: the score is that of the scoring oracle."""
    rng = np.random.default_rng(13)
    q = rng.standard_normal((4, 5, 128)).astype(np.float32)
    k = rng.standard_normal((2, 300, 128)).astype(np.float32)
    if dtype == "bf16":
        q = (q.view(np.uint32) >> 16).astype(np.uint16)
        k = (k.view(np.uint32) >> 16).astype(np.uint16)
    want, _, _ = oracle.scores(q, k)
    for chunk, fe in ((300, 0), (150, 0), (148, 4), (1000, 0)):
        np.testing.assert_allclose(oracle.scores_dca(q, k, chunk, fe), want, rtol=1e-12)
    wmax, _, _ = oracle.scores(q, k, mode=oracle.MODE_MAX)
    np.testing.assert_allclose(oracle.scores_dca(q, k, 150, 0, mode_max=True), wmax, rtol=1e-12)


def test_round_bf16_matches_library_conversion():
    rng = np.random.default_rng(14)
    x = np.concatenate([rng.standard_normal(4096) * np.exp(rng.uniform(-20, 20, 4096)),
                        [1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -1.0 - 2.0 ** -8, 0.0, 255.5, 256.5]]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(oracle.round_bf16(x.astype(np.float64)), want)
    # ties go to the even neighbour
    assert oracle.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert oracle.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # straight from fp64, no detour over fp32: just above the tie goes up although fp32 would see the tie
    assert oracle.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1.0 + 2.0 ** -7


def test_bf16_query_rounding_is_applied_to_turned_chunks_only():
    rng = np.random.default_rng(15)
    q = (rng.standard_normal((2, 2, 16)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    k = (rng.standard_normal((1, 40, 16)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    qw = (q.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    kw = (k.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    got = oracle.logits_dca(q, k, 10, 0, base=100.0)
    freq = oracle.default_inv_freq(16, 100.0)
    # chunks 0,1 turned by 20 and 10 tokens, chunks 2,3 untouched
    for c, D in enumerate((20, 10, 0, 0)):
        qc = oracle.rotate(qw, -D, freq) if D else qw
        if D:
            qc = torch.from_numpy(qc.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
        want = np.einsum("hid,td->hit", qc, kw[0, 10 * c:10 * c + 10]) / 4.0
        # (the library conversion goes over fp32; on these seeded values no element sits close enough to a
        # bf16 tie for that detour to matter)
        assert np.abs(got[:, :, 10 * c:10 * c + 10] - want).max() < 1e-14
