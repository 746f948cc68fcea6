"""agq_gemm_w4a8_static (the linear layer on the library's fixed workspace, for callers that cannot allocate)
against agq_gemm_w4a8 on a caller workspace: same kernels, so accumulators and fp16 outputs must be identical bit
for bit; and against the oracle, to the bar of the other GEMM tests.  Two calls in a row share the array, the
second with a smaller input."""
from __future__ import annotations

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2312_05693_amd import synth  # noqa: E402


@pytest.fixture(scope="module")
def agq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2312_05693_amd import binding
    binding.lib()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_static_workspace_two_calls_in_a_row(agq, oracle):
    # (M, K, N): a K split with partial tiles behind the codes, then a smaller call that leaves stale bytes of the
    # first in the array, then a weight-streaming call (no workspace at all) and a many-tile call without a split
    cases = [(600, 2048, 384, 31), (300, 2048, 256, 32), (5, 512, 48, 33), (1000, 768, 1024, 34)]
    inputs = []
    for (M, K, N, seed) in cases:
        x = synth.make_activation(M, K, 4, seed)
        wq, sw = synth.make_weight_q4(N, K, seed)
        e = oracle.calibrate_act_exp(x, 8)
        inputs.append((dev(x), e, agq.pack_w4(dev(wq)), dev(sw), oracle.linear_w4(x, 8, e, 0, wq, sw)))
    # the first two cases do split K when given the room (that is what puts partial tiles into the array)
    for (M, K, N, _) in cases[:2]:
        assert agq.gemm_workspace_bytes(M, N, K) > agq.gemm_workspace_bytes(M, 0, K)
        assert agq.gemm_workspace_bytes(M, N, K) <= agq.lib().agq_gemm_workspace_bytes(2048, 0, 11008)
    outs = []
    for (M, K, N, _), (xd, e, blob, swd, _) in zip(cases, inputs):     # back to back, no synchronisation between
        y = torch.empty((M, N), dtype=torch.float16, device="cuda")
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
        agq.gemm_w4a8_static(xd, e, blob, swd, N, K, y, acc_out=acc)
        outs.append((y, acc))
    torch.cuda.synchronize()
    for (M, K, N, _), (xd, e, blob, swd, (acc_w, y_w)), (y, acc) in zip(cases, inputs, outs):
        acc_ref = torch.empty((M, N), dtype=torch.int32, device="cuda")
        y_ref = agq.gemm_w4a8(xd, e, blob, swd, N, K, acc_out=acc_ref)
        torch.cuda.synchronize()
        assert torch.equal(acc, acc_ref), (M, K, N)
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), (M, K, N)
        assert np.array_equal(acc.cpu().numpy().astype(np.int64), acc_w), (M, K, N)
        got, want = y.cpu().numpy().astype(np.float64), y_w.astype(np.float64)
        assert np.all(np.abs(got - want) <= 1e-3 * np.abs(want) + 2.0 ** -24), (M, K, N)


def test_static_workspace_rejects_what_does_not_fit(agq):
    x = torch.empty(16, dtype=torch.float16, device="cuda")          # never read: the size check comes first
    p = x.data_ptr()
    st = agq.lib().agq_gemm_w4a8_static(p, 0, 4096, 16384, 16384, 0, 0, p, p, 16, p, 16, None, None)   # 64 MiB of codes
    assert st == agq.AGQ_ESIZE
    assert agq.lib().agq_status_string(st) == b"workspace too small"
