"""Helpers for the GPU parity tests: move bf16 bit patterns to and from device memory (torch is
used for allocation and streams only) and call the three products through the C ABI."""
from __future__ import annotations

import numpy as np
import torch

import paper_2305_13525_amd as axo

REL_FRO_TOL = 2e-3      # relative Frobenius error against the fp64 oracle
PER_ELEM_TOL = 1e-2     # |C - O| <= 1e-2 * max_c |O[r, c]|
# The 2e-3 Frobenius bound is a statement about the RMS of round-to-nearest-even bf16 rounding
# (about 1.66e-3 of the value) and only holds once enough elements average out: a single
# correctly rounded element can be off by the unit roundoff 2^-8 = 3.9e-3.  It is therefore
# applied to outputs of at least SMALL_OUTPUT elements.  The statement that holds at any size, and
# is applied at every size, is the element-wise one: every output is within ONE bf16 step of the
# oracle value rounded once to bf16, unless it is so close to zero that the fp32 accumulation error
# (FAR_ABS of the row's largest magnitude: the benchmark's sums of up to 16384 products carry about
# 1e-5 of it) spans more than a bf16 step there.
SMALL_OUTPUT = 4096
FAR_ABS = 1e-4


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


def assert_close(oracle_mod, cand_bits, ref, what="", fro=None, per_elem=PER_ELEM_TOL, one_step=None):
    """`fro` overrides the Frobenius bound for results that went through more than one rounding (sums of
    bf16 partial results); the one-step gate is for singly rounded results and is then off by default."""
    if one_step is None:
        one_step = fro is None
    cand_bits = np.ascontiguousarray(cand_bits)
    r = oracle_mod.compare_bf16(cand_bits, ref, per_elem)
    assert r["n_nonfinite"] == 0, (what, r)
    steps = oracle_mod.ulp_distance_bf16(cand_bits, ref)
    err = np.abs((cand_bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64) - ref)
    row_max = np.max(np.abs(ref), axis=1, keepdims=True) if ref.size else np.zeros((ref.shape[0], 1))
    r["n_beyond_1_step"] = int(np.count_nonzero(steps > 1))          # reported
    r["n_far"] = int(np.count_nonzero((steps > 1) & (err > FAR_ABS * row_max)))   # gated
    assert r["n_far"] == 0 or not one_step, (what, r)
    if fro is not None or ref.size >= SMALL_OUTPUT:
        assert r["rel_fro"] <= (REL_FRO_TOL if fro is None else fro), (what, r)
    assert r["n_bad"] == 0, (what, r)
    return r
