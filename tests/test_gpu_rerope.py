"""GPU parity of the DCA re-RoPE of the key cache (Section 3.3, second DCA equation): the HIP kernel,
called through the C ABI, against the fp64 oracle on the same seeded caches."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2508_17892_amd as il
from parity import score_errors, to_device

pytestmark = pytest.mark.gpu


def _announce(msg):
    print(f"[case] {msg}", flush=True)


def _check(got_dev, k_host, exact, dtype):
    """got: device result; exact: fp64 oracle.  fp32 caches: rotation error of a few fp32 ulps of the pair.
    bf16 caches: that plus half a bf16 ulp of the value, and all but a sliver of the elements must carry
    exactly the oracle's value rounded to nearest even."""
    src = inputs.as_float(k_host).astype(np.float64)
    # an element's pair is bounded by twice the row's largest magnitude, whatever the pairing
    pair_mag = np.abs(src).max(axis=-1, keepdims=True) * 2.0 + np.zeros_like(src)
    if dtype == "bf16":
        got = inputs.bf16_bits_to_f32(got_dev.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
        tol = np.abs(exact) * 2.0 ** -8 * 1.001 + 1e-6 * pair_mag   # half a bf16 ulp is at most 2^-8 of the value
        assert (np.abs(got - exact) <= tol).all(), float((np.abs(got - exact) / tol).max())
        want_bits = inputs.f32_to_bf16_bits(exact.astype(np.float32))
        got_bits = got_dev.view(torch.int16).cpu().numpy().view(np.uint16)
        assert (want_bits != got_bits).mean() < 2e-3
    else:
        got = got_dev.cpu().numpy().astype(np.float64)
        tol = 1e-6 * pair_mag
        assert (np.abs(got - exact) <= tol).all(), float((np.abs(got - exact) / tol).max())
    return got


CASES = [
    # name, Hkv, L, chunk, first_extra, dtype, pairing, base
    ("paper_default_bf16", 2, 9000, 1024, 4, "bf16", il.ILRE_ROPE_HALF, 500000.0),
    ("interleaved_bf16", 2, 5000, 512, 4, "bf16", il.ILRE_ROPE_INTERLEAVED, 10000.0),
    ("f32_half", 1, 3000, 100, 0, "f32", il.ILRE_ROPE_HALF, 10000.0),
    ("f32_interleaved", 2, 2500, 333, 7, "f32", il.ILRE_ROPE_INTERLEAVED, 10000.0),
    ("single_chunk_is_a_copy", 2, 700, 1024, 4, "bf16", il.ILRE_ROPE_HALF, 10000.0),
    ("two_chunks_are_a_copy", 1, 1500, 1024, 4, "bf16", il.ILRE_ROPE_HALF, 10000.0),
    ("chunk_smaller_than_a_slice", 1, 2000, 37, 3, "bf16", il.ILRE_ROPE_HALF, 10000.0),
    ("long_distances", 1, 300000, 1024, 4, "bf16", il.ILRE_ROPE_HALF, 500000.0),
    ("one_token", 1, 1, 8, 0, "f32", il.ILRE_ROPE_HALF, 10000.0),
]


@pytest.mark.parametrize("name,Hkv,L,chunk,extra,dtype,pairing,base", CASES, ids=[c[0] for c in CASES])
def test_rerope_against_oracle(name, Hkv, L, chunk, extra, dtype, pairing, base):
    _announce(f"rerope {name} Hkv={Hkv} L={L} chunk={chunk} extra={extra} {dtype} pairing={pairing}")
    inp = inputs.custom(L=L, Lq=4, Hq=Hkv, Hkv=Hkv, d=128, dtype=dtype, seed=len(name))
    exact = oracle.rerope_keys(inp.k, chunk, extra, base, pairing=pairing)
    k = to_device(inp.k)
    out = il.ilre_rerope_keys(k, chunk, extra, rope_base=base, pairing=pairing)
    torch.cuda.synchronize()
    _check(out, inp.k, exact, dtype)
    # the last two chunks are copied bit for bit
    bounds = oracle.chunk_bounds(L, chunk, extra)
    start = bounds[-2][0] if len(bounds) >= 2 else 0
    assert torch.equal(out[:, start:, :], k[:, start:, :])
    # in place gives the same bits
    k2 = k.clone()
    il.ilre_rerope_keys(k2, chunk, extra, rope_base=base, pairing=pairing, out=k2)
    torch.cuda.synchronize()
    assert torch.equal(k2, out)


def test_rerope_token_major_and_scaled_frequencies():
    _announce("rerope token-major cache, caller's frequency table")
    inp = inputs.custom(L=4000, Lq=4, Hq=2, Hkv=2, d=128, dtype="bf16", seed=21)
    freq = oracle.default_inv_freq(128, 500000.0)
    freq = np.where(freq < 1e-3, freq / 8.0, freq)          # low frequencies scaled down, as length-extended models do
    exact = oracle.rerope_keys(inp.k, 512, 4, inv_freq=freq)
    k = to_device(inp.k)
    k_tm = k.permute(1, 0, 2).contiguous().permute(1, 0, 2)  # storage [L, Hkv, d]
    out = il.ilre_rerope_keys(k_tm, 512, 4, inv_freq=freq.tolist())
    torch.cuda.synchronize()
    assert out.stride() == k_tm.stride()
    _check(out.contiguous(), inp.k, exact, "bf16")


def test_recall_on_a_reroped_cache():
    """DCA on: re-RoPE, then the recall step.  fp32 so that both sides feed the scoring the same keys up to
    fp32 rounding of the rotation."""
    _announce("rerope then recall (f32)")
    inp = inputs.custom(L=6000, Lq=16, Hq=8, Hkv=2, d=128, dtype="f32", n_spans=2, span_len=(32, 32), seed=9)
    k_rot = oracle.rerope_keys(inp.k, 1024, 4, 500000.0).astype(np.float32)
    want, _, _ = oracle.scores(inp.q, k_rot)
    q, k = to_device(inp.q), to_device(inp.k)
    k_dev = il.ilre_rerope_keys(k, 1024, 4, rope_base=500000.0)
    _, got = il.ilre_recall(q, k_dev, 256, (3, 7))
    torch.cuda.synchronize()
    bad, worst = score_errors(got.cpu().numpy(), want)
    assert bad == 0, worst
