"""Helpers for the GPU parity tests: move bf16 bit patterns to and from device memory (torch is
used for allocation and streams only) and call the three products through the C ABI."""
from __future__ import annotations

import numpy as np
import torch

import paper_2305_13525_amd as axo

REL_FRO_TOL = 2e-3      # relative Frobenius error against the fp64 oracle
PER_ELEM_TOL = 1e-2     # |C - O| <= 1e-2 * max_c |O[r, c]|
# The 2e-3 Frobenius bound is a statement about the RMS of round-to-nearest-even bf16 rounding
# (about 1.66e-3 of the value) and only holds once enough elements average out.  A single
# correctly rounded element can be off by the unit roundoff 2^-8 = 3.9e-3, so outputs with
# fewer than SMALL_OUTPUT elements are held to that hard bound (plus 2^-12 for fp32 summation).
SMALL_OUTPUT = 4096
SMALL_FRO_TOL = 2.0 ** -8 + 2.0 ** -12


def fro_tol(n_elems: int) -> float:
    return REL_FRO_TOL if n_elems >= SMALL_OUTPUT else SMALL_FRO_TOL


def to_dev(bits: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(bits, dtype=np.uint16)
    return torch.from_numpy(a.view(np.int16)).to("cuda:0")


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().view(np.uint16)


def empty_dev(rows: int, cols: int, fill: int = 0x7FC0) -> torch.Tensor:
    """Output buffer pre-filled with a bf16 NaN pattern so unwritten elements are noticed."""
    return torch.full((rows, cols), fill, dtype=torch.int16, device="cuda:0")


def stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def ld(t: torch.Tensor) -> int:
    return t.stride(0) if t.dim() == 2 else t.numel()


def ws_for(p, op):
    n = axo.axo_workspace_bytes(p, op)
    if n == 0:
        return None, None, 0
    buf = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    return buf, buf.data_ptr(), n


def run_fwd(p, X, W, Y, bias=None, epilogue=0):
    buf, wp, wn = ws_for(p, axo.AXO_OP_FWD)
    axo.axo_fc_fwd(p, X.data_ptr(), ld(X), W.data_ptr(), ld(W), None if bias is None else bias.data_ptr(),
                   epilogue, Y.data_ptr(), ld(Y), wp, wn, stream())
    return buf


def run_dgrad(p, dY, W, dX):
    buf, wp, wn = ws_for(p, axo.AXO_OP_DGRAD)
    axo.axo_fc_dgrad(p, dY.data_ptr(), ld(dY), W.data_ptr(), ld(W), dX.data_ptr(), ld(dX), wp, wn, stream())
    return buf


def run_wgrad(p, X, dY, dW):
    buf, wp, wn = ws_for(p, axo.AXO_OP_WGRAD)
    axo.axo_fc_wgrad(p, X.data_ptr(), ld(X), dY.data_ptr(), ld(dY), dW.data_ptr(), ld(dW), wp, wn, stream())
    return buf


def trio(p, Xb, Wb, dYb, bias_b=None, epilogue=0):
    """Upload bit patterns, run fwd/dgrad/wgrad through the C ABI, return bf16 bit arrays."""
    M, Kl = Xb.shape
    Nl = Wb.shape[1]
    X, W, dY = to_dev(Xb), to_dev(Wb), to_dev(dYb)
    bias = None if bias_b is None else to_dev(bias_b)
    Y, dX, dW = empty_dev(M, Nl), empty_dev(M, Kl), empty_dev(Kl, Nl)
    keep = [run_fwd(p, X, W, Y, bias, epilogue), run_dgrad(p, dY, W, dX), run_wgrad(p, X, dY, dW)]
    torch.cuda.synchronize()
    del keep
    return to_host(Y), to_host(dX), to_host(dW)


def assert_close(oracle_mod, cand_bits, ref, what="", fro=None, per_elem=PER_ELEM_TOL):
    r = oracle_mod.compare_bf16(np.ascontiguousarray(cand_bits), ref, per_elem)
    assert r["n_nonfinite"] == 0, (what, r)
    assert r["rel_fro"] <= (fro_tol(ref.size) if fro is None else fro), (what, r)
    assert r["n_bad"] == 0, (what, r)
    return r
