"""fp64 CPU oracle of the 3D-tensor-parallel FC shard GEMMs -- TEST INFRASTRUCTURE ONLY.

Nothing in the product package may import this.  Only tests/, the smoke check and the
benchmark's cpu_baseline leg call it.  It is independent of the HIP library: no shared
code, headers or tables; inputs arrive as bf16 bit patterns (uint16 numpy arrays).

The arithmetic lives in axo_oracle.c (plain loops, fp64).  This file marshals numpy
arrays into it and states, in numpy slicing, how the global matrices of a layer are cut
over the Gx x Gy x Gz grid (paper Section 3.2: 2D decompositions of I and W mapped to
orthogonal planes of the grid; Algorithm 1 for which axis each partial result is summed
over).  Axis naming follows the benchmark's convention: the reduction dimension K of the
forward product is split over Gx, the output features N over Gy, the tokens T over Gz.
With `transposed=True` the roles of the X and Y axes swap (Section 3.2, "Parallelizing
an entire network": every second layer), which is Algorithm 1 exactly as printed.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

EPI_NONE, EPI_BIAS, EPI_BIAS_GELU_TANH, EPI_BIAS_GELU_ERF = 0, 1, 2, 3

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        i64, p = ctypes.c_int64, ctypes.c_void_p
        L.oracle_fc_fwd.argtypes = [p, i64, p, i64, p, ctypes.c_int, i64, i64, i64, p, i64, p]
        L.oracle_fc_dgrad.argtypes = [p, i64, p, i64, i64, i64, i64, p, i64, p]
        L.oracle_fc_wgrad.argtypes = [p, i64, p, i64, i64, i64, i64, p, i64, p]
        L.oracle_compare_bf16.argtypes = [p, i64, p, i64, i64, ctypes.c_double, p]
        L.oracle_gelu_erf.argtypes = [ctypes.c_double]
        L.oracle_gelu_erf.restype = ctypes.c_double
        L.oracle_gelu_tanh.argtypes = [ctypes.c_double]
        L.oracle_gelu_tanh.restype = ctypes.c_double
        L.oracle_num_threads.restype = ctypes.c_int
        for name in ("oracle_dgelu_erf", "oracle_dgelu_tanh"):
            getattr(L, name).argtypes = [ctypes.c_double]
            getattr(L, name).restype = ctypes.c_double
        L.oracle_fc_dgrad_act.argtypes = [p, i64, p, i64, p, i64, ctypes.c_int, i64, i64, i64, p, i64, p]
        L.oracle_bias_grad.argtypes = [p, i64, i64, i64, p]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _u16(a: np.ndarray) -> np.ndarray:
    assert a.dtype == np.uint16 and a.ndim == 2 and a.strides[1] == 2, "bf16 bits, 2-D, unit column stride"
    assert a.strides[0] % 2 == 0 and a.strides[0] >= 0
    return a


def _ld(a: np.ndarray) -> int:
    return a.strides[0] // 2 if a.shape[0] > 1 else max(a.shape[1], a.strides[0] // 2)


def _rows(rows: Optional[Sequence[int]], limit: int):
    if rows is None:
        return None, limit, None
    r = np.ascontiguousarray(rows, dtype=np.int64)
    assert r.ndim == 1 and (r.size == 0 or (r.min() >= 0 and r.max() < limit))
    return r, int(r.size), r.ctypes.data


def fc_fwd(X: np.ndarray, W: np.ndarray, bias: Optional[np.ndarray] = None, epilogue: int = EPI_NONE,
           rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """Y = X . W (+bias, activation) in fp64; Algorithm 1, forward local product."""
    X, W = _u16(X), _u16(W)
    M, Kl = X.shape
    assert W.shape[0] == Kl
    Nl = W.shape[1]
    keep, n_rows, rp = _rows(rows, M)
    out = np.empty((n_rows, Nl), dtype=np.float64)
    bp = None
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.uint16)
        assert bias.shape == (Nl,)
        bp = bias.ctypes.data
    rc = lib().oracle_fc_fwd(X.ctypes.data, _ld(X), W.ctypes.data, _ld(W), bp, int(epilogue),
                             M, Kl, Nl, rp, n_rows, out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_fc_fwd: epilogue needs a bias")
    return out


def fc_dgrad(dY: np.ndarray, W: np.ndarray, rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """dX = dY . W^T in fp64; Algorithm 1, backward function, first product."""
    dY, W = _u16(dY), _u16(W)
    M, Nl = dY.shape
    Kl = W.shape[0]
    assert W.shape[1] == Nl
    keep, n_rows, rp = _rows(rows, M)
    out = np.empty((n_rows, Kl), dtype=np.float64)
    lib().oracle_fc_dgrad(dY.ctypes.data, _ld(dY), W.ctypes.data, _ld(W), M, Kl, Nl, rp, n_rows, out.ctypes.data)
    return out


def fc_wgrad(X: np.ndarray, dY: np.ndarray, rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """dW = X^T . dY in fp64; Algorithm 1, backward function, second product.  `rows` index dW's rows."""
    X, dY = _u16(X), _u16(dY)
    M, Kl = X.shape
    assert dY.shape[0] == M
    Nl = dY.shape[1]
    keep, n_rows, rp = _rows(rows, Kl)
    out = np.empty((n_rows, Nl), dtype=np.float64)
    lib().oracle_fc_wgrad(X.ctypes.data, _ld(X), dY.ctypes.data, _ld(dY), M, Kl, Nl, rp, n_rows, out.ctypes.data)
    return out


def fc_dgrad_act(dY: np.ndarray, W: np.ndarray, pre: np.ndarray, act: int,
                 rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """(dY . W^T) * act'(pre) in fp64: the data gradient taken through the activation of the layer below."""
    dY, W, pre = _u16(dY), _u16(W), _u16(pre)
    M, Nl = dY.shape
    Kl = W.shape[0]
    assert W.shape[1] == Nl and pre.shape == (M, Kl)
    keep, n_rows, rp = _rows(rows, M)
    out = np.empty((n_rows, Kl), dtype=np.float64)
    rc = lib().oracle_fc_dgrad_act(dY.ctypes.data, _ld(dY), W.ctypes.data, _ld(W), pre.ctypes.data, _ld(pre), int(act),
                                   M, Kl, Nl, rp, n_rows, out.ctypes.data)
    assert rc == 0
    return out


def bias_grad(dY: np.ndarray) -> np.ndarray:
    """Column sums of dY in fp64: the bias gradient."""
    dY = _u16(dY)
    M, Nl = dY.shape
    out = np.empty(Nl, dtype=np.float64)
    lib().oracle_bias_grad(dY.ctypes.data, _ld(dY), M, Nl, out.ctypes.data)
    return out


def dgelu_tanh(x: float) -> float:
    return float(lib().oracle_dgelu_tanh(float(x)))


def dgelu_erf(x: float) -> float:
    return float(lib().oracle_dgelu_erf(float(x)))


def gelu_tanh(x: float) -> float:
    return float(lib().oracle_gelu_tanh(float(x)))


def gelu_erf(x: float) -> float:
    return float(lib().oracle_gelu_erf(float(x)))


def compare_bf16(cand_bits: np.ndarray, ref: np.ndarray, per_elem_tol: float = 1e-2) -> dict:
    """Error of a bf16 candidate against the fp64 oracle block: relative Frobenius error and
    the per-element bound |C-O| <= tol * max_c |O[r,c]| (row infinity norm of the oracle row)."""
    cand_bits = _u16(cand_bits)
    ref = np.ascontiguousarray(ref, dtype=np.float64)
    assert cand_bits.shape == ref.shape
    res = np.zeros(4, dtype=np.float64)
    lib().oracle_compare_bf16(cand_bits.ctypes.data, _ld(cand_bits), ref.ctypes.data, ref.shape[0], ref.shape[1],
                              float(per_elem_tol), res.ctypes.data)
    return {"rel_fro": float(res[0]), "max_rel_row": float(res[1]), "n_bad": int(res[2]), "n_nonfinite": int(res[3])}


def rne_bf16_bits(ref: np.ndarray) -> np.ndarray:
    """fp64 values rounded once, to nearest with ties to even, to bf16 bit patterns (the rounding the
    benchmark's north star asks of the store).  fp64 -> fp32 is done with round-to-odd (truncate
    towards zero, then set the last mantissa bit if anything was lost), which makes the second
    rounding, fp32 -> bf16 nearest-even on the bit pattern, equal to a single direct rounding.
    Finite inputs inside the fp32 range."""
    x = np.ascontiguousarray(ref, dtype=np.float64)
    with np.errstate(over="ignore", under="ignore"):
        f = x.astype(np.float32)
    fd = f.astype(np.float64)
    inexact = fd != x
    away = np.abs(fd) > np.abs(x)                      # the nearest fp32 lies beyond x: step back towards zero
    t = np.where(inexact & away, np.nextafter(f, np.float32(0.0)), f).astype(np.float32)
    u = t.view(np.uint32) | inexact.astype(np.uint32)  # round to odd
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def ulp_distance_bf16(cand_bits: np.ndarray, ref: np.ndarray) -> np.ndarray:
    """How many bf16 values lie between each candidate and the oracle value rounded once to bf16
    (0 = the correctly rounded result; +0 and -0 count as the same value).  Finite values."""
    def ordinal(b):
        b = np.asarray(b, dtype=np.uint16).astype(np.int32)
        return np.where(b < 0x8000, b, -(b & 0x7FFF))
    return np.abs(ordinal(cand_bits) - ordinal(rne_bf16_bits(ref)))


# ---------------------------------------------------------------------------
# Grid decomposition (Section 3.2; Algorithm 1 for the reduce axes)
# ---------------------------------------------------------------------------
def _axes(grid: Tuple[int, int, int], coord: Tuple[int, int, int], transposed: bool):
    gx, gy, gz = grid
    ix, iy, iz = coord
    if transposed:  # K over Gy, N over Gx -- Algorithm 1 as printed (I_{k,j}, W_{j,i})
        return (gy, iy), (gx, ix), (gz, iz)
    return (gx, ix), (gy, iy), (gz, iz)  # K over Gx, N over Gy, T over Gz


def shard_slices(T: int, K: int, N: int, grid, coord, transposed: bool = False):
    """(rows of X/Y, cols of X = rows of W, cols of W/Y) owned by GPU g_{coord}."""
    (gk, ik), (gn, i_n), (gt, it) = _axes(grid, coord, transposed)
    assert T % gt == 0 and K % gk == 0 and N % gn == 0
    m, kl, nl = T // gt, K // gk, N // gn
    return slice(it * m, (it + 1) * m), slice(ik * kl, (ik + 1) * kl), slice(i_n * nl, (i_n + 1) * nl)


def shards(Xg: np.ndarray, Wg: np.ndarray, dYg: np.ndarray, grid, coord, transposed: bool = False):
    """Views (no copy) of the blocks I_{k,j}, W_{j,i}, dO_{k,i} of GPU g_{coord} inside the global tensors."""
    T, K = Xg.shape
    N = Wg.shape[1]
    rt, rk, rn = shard_slices(T, K, N, grid, coord, transposed)
    return Xg[rt, rk], Wg[rk, rn], dYg[rt, rn]


def assemble_from_shards(Xg, Wg, dYg, grid, transposed: bool = False, fwd=fc_fwd, dgrad=fc_dgrad, wgrad=fc_wgrad):
    """Run the three local products on every GPU of the grid, one after another, and combine
    them the way the collectives of Algorithm 1 would: the forward partials are summed over
    the axis that splits K and placed at (T-block, N-block); the dgrad partials are summed over
    the axis that splits N; the wgrad partials are summed over Z.  `fwd/dgrad/wgrad` take bf16
    bit blocks and return fp64 blocks (default: this oracle)."""
    T, K = Xg.shape
    N = Wg.shape[1]
    gx, gy, gz = grid
    Y = np.zeros((T, N))
    dX = np.zeros((T, K))
    dW = np.zeros((K, N))
    for iz in range(gz):
        for iy in range(gy):
            for ix in range(gx):
                c = (ix, iy, iz)
                rt, rk, rn = shard_slices(T, K, N, grid, c, transposed)
                Xs, Ws, dYs = Xg[rt, rk], Wg[rk, rn], dYg[rt, rn]
                Y[rt, rn] += fwd(Xs, Ws)
                dX[rt, rk] += dgrad(dYs, Ws)
                dW[rk, rn] += wgrad(Xs, dYs)
    return Y, dX, dW
