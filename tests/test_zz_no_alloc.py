"""ilre_row_stats_static, the entry point that allocates nothing (its scratch is a buffer built into the
library): bit-identical to ilre_row_stats through the C ABI, on two calls in a row that share the buffer,
the second on a smaller input, then the first shape again."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import paper_2508_17892_amd as il
from parity import to_device

pytestmark = pytest.mark.gpu


def _case(L, Lq, Hq, Hkv, dtype, seed):
    inp = inputs.custom(L=L, Lq=Lq, Hq=Hq, Hkv=Hkv, d=128, dtype=dtype, n_spans=2, span_len=(8, 24), channel_scale=True,
                        seed=seed)
    return inp, to_device(inp.q), to_device(inp.k)


def test_row_stats_static_matches_row_stats_on_consecutive_calls():
    print("[case] no-alloc row statistics: 20000x(8x96) bf16, then 3001x(4x10) bf16, then f32, then the first again",
          flush=True)
    cases = [_case(20000, 96, 8, 2, "bf16", 51), _case(3001, 10, 4, 2, "bf16", 52), _case(1500, 24, 8, 4, "f32", 53)]
    cases.append(cases[0])
    outs = [(torch.empty(i.q.shape[0] * i.q.shape[1], dtype=torch.float32, device="cuda"),
             torch.empty(i.q.shape[0] * i.q.shape[1], dtype=torch.float32, device="cuda")) for i, _, _ in cases]
    torch.cuda.synchronize()
    held = torch.cuda.memory_allocated()
    # back to back on one stream, no synchronisation in between: the calls share the library's buffer in order
    for (inp, q, k), (ref, sumexp) in zip(cases, outs):
        ref.fill_(float("nan"))
        sumexp.fill_(float("nan"))
        il.ilre_row_stats_static(q, k, ref, sumexp)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == held
    for n, ((inp, q, k), (ref, sumexp)) in enumerate(zip(cases, outs)):
        want_ref, want_sum = il.ilre_row_stats(q, k)
        torch.cuda.synchronize()
        assert torch.equal(ref, want_ref) and torch.equal(sumexp, want_sum), f"call {n}"
        # and, as for the existing entry point, the oracle's log-sum-exp
        _, omax, osum = oracle.scores(inp.q, inp.k)
        got = ref.cpu().numpy().astype(np.float64) + np.log(sumexp.cpu().numpy().astype(np.float64))
        np.testing.assert_allclose(got, omax + np.log(osum), rtol=0, atol=2e-4)
    # the exact-maximum form through the same buffer
    inp, q, k = cases[1]
    ref, sumexp = outs[1]
    il.ilre_row_stats_static(q, k, ref, sumexp, flags=il.ILRE_FLAG_EXACT_ROW_MAX)
    want_ref, want_sum = il.ilre_row_stats(q, k, flags=il.ILRE_FLAG_EXACT_ROW_MAX)
    torch.cuda.synchronize()
    assert torch.equal(ref, want_ref) and torch.equal(sumexp, want_sum)
