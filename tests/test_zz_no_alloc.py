"""The allocation-free entry point axo_bias_grad_static against axo_bias_grad_ws (same kernel, the
scratch memory in a fixed device array instead of a caller workspace): two calls in a row through the
C ABI, the second on a smaller input, each bit for bit equal to the workspace form and within fp32
summation error of the fp64 oracle.  Host part: argument errors and the limit, without a device."""
import numpy as np
import pytest

import axo_synth as syn
import oracle
import paper_2305_13525_amd as axo

torch = pytest.importorskip("torch")


def P(M, Nl):
    return axo.Problem.make((1, 1, 1), (0, 0, 0), M, 8, Nl)


def test_static_entry_point_host_checks():
    A, B = 0x10000, 1 << 40
    assert axo.axo_bias_grad_static_limit() == 256 * 1024
    p = P(4096, 6144)
    assert axo.axo_bias_grad_workspace_bytes(p) <= axo.axo_bias_grad_static_limit()
    f = lambda **kw: axo.axo_bias_grad_static(**{**dict(p=p, dY=A, lddy=6144, db=B, accumulate=0, check=False), **kw})
    assert f(db=None) == -4 and f(lddy=6136) == -6 and f(accumulate=2) == -11 and f(db=B + 2) == -5
    assert f(db=A + 64) == -11                                            # db inside dY
    assert axo.axo_bias_grad_static(P(64, 0), A, 8, B, 0, check=False) == 0   # nothing to do: no device needed
    assert axo.axo_status_string(-13).startswith("problem needs more scratch")
    # the widest slicing any shape gets stays inside the array: strips of 64 columns, S slices
    worst = max(axo.axo_bias_grad_workspace_bytes(P(1 << 20, n)) for n in range(64, 70000, 64))
    assert 0 < worst <= axo.axo_bias_grad_static_limit()


@pytest.mark.gpu
def test_static_entry_point_matches_workspace_form_twice():
    import gpu_util as gu
    for M, Nl in ((4096, 6144), (1000, 520)):                     # the second call is the smaller one
        dYb = syn.normal_bf16(28, 0, (M, Nl), 1.0)
        dY = gu.to_dev(dYb)
        p = P(M, Nl)
        nws = axo.axo_bias_grad_workspace_bytes(p)
        assert nws > 0                                            # both shapes really use scratch memory
        ws = torch.zeros(nws, dtype=torch.uint8, device="cuda:0")
        want = torch.full((Nl,), float("nan"), dtype=torch.float32, device="cuda:0")
        got = torch.full((Nl,), float("nan"), dtype=torch.float32, device="cuda:0")
        axo.axo_bias_grad_ws(p, dY.data_ptr(), Nl, want.data_ptr(), 0, ws.data_ptr(), nws, gu.stream())
        axo.axo_bias_grad_static(p, dY.data_ptr(), Nl, got.data_ptr(), 0, gu.stream())
        torch.cuda.synchronize()
        assert torch.equal(got, want), (M, Nl)
        ref = oracle.bias_grad(dYb)
        assert np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref)) <= 4e-6 * np.sqrt(M) * 4 + 1e-6
        # accumulate on top, still through the static scratch
        axo.axo_bias_grad_static(p, dY.data_ptr(), Nl, got.data_ptr(), 1, gu.stream())
        axo.axo_bias_grad_ws(p, dY.data_ptr(), Nl, want.data_ptr(), 1, ws.data_ptr(), nws, gu.stream())
        torch.cuda.synchronize()
        assert torch.equal(got, want), (M, Nl, "accumulate")
