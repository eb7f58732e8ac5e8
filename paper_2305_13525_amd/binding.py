"""ctypes binding of libaxo.so: argument marshalling only.

Function names and argument order mirror include/axo.h.  Matrices are passed as raw device
addresses (`tensor.data_ptr()`), streams as raw `hipStream_t` values
(`torch.cuda.current_stream().cuda_stream`).  Nothing here computes: if the library is missing
the import of a symbol fails loudly; there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libaxo.so")

AXO_EPI_NONE, AXO_EPI_BIAS, AXO_EPI_BIAS_GELU_TANH, AXO_EPI_BIAS_GELU_ERF = 0, 1, 2, 3
AXO_OP_FWD, AXO_OP_DGRAD, AXO_OP_WGRAD = 0, 1, 2
AXO_ROUTE_NONE, AXO_ROUTE_TILED, AXO_ROUTE_COVERED, AXO_ROUTE_INTERIOR_STRIPS, AXO_ROUTE_GENERAL = 0, 1, 2, 3, 4


class AxoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({axo_status_string(status)})")


class Problem(ctypes.Structure):
    """axo_problem_t: grid, this GPU's coordinate, global sizes, axis mapping."""
    _fields_ = [("Gx", ctypes.c_int32), ("Gy", ctypes.c_int32), ("Gz", ctypes.c_int32),
                ("ix", ctypes.c_int32), ("iy", ctypes.c_int32), ("iz", ctypes.c_int32),
                ("T", ctypes.c_int64), ("K", ctypes.c_int64), ("N", ctypes.c_int64),
                ("transposed", ctypes.c_int32), ("reserved", ctypes.c_int32)]

    @classmethod
    def make(cls, grid: Tuple[int, int, int], coord: Tuple[int, int, int], T: int, K: int, N: int,
             transposed: int = 0) -> "Problem":
        return cls(grid[0], grid[1], grid[2], coord[0], coord[1], coord[2], T, K, N, transposed, 0)


class Layer(ctypes.Structure):
    """axo_layer_t: one FC layer of a chain with the caller's device buffers."""
    _fields_ = [("p", Problem), ("epilogue", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("X", ctypes.c_void_p), ("ldx", ctypes.c_int64),
                ("W", ctypes.c_void_p), ("ldw", ctypes.c_int64),
                ("bias", ctypes.c_void_p),
                ("Y", ctypes.c_void_p), ("ldy", ctypes.c_int64),
                ("dY", ctypes.c_void_p), ("lddy", ctypes.c_int64),
                ("dX", ctypes.c_void_p), ("lddx", ctypes.c_int64),
                ("dW", ctypes.c_void_p), ("lddw", ctypes.c_int64)]


class LayerExt(ctypes.Structure):
    """axo_layer_ext_t: a layer plus the optional backward-side extras of axo_layer_step_ext."""
    _fields_ = [("layer", Layer),
                ("pre", ctypes.c_void_p), ("ldpre", ctypes.c_int64),
                ("dW32", ctypes.c_void_p), ("lddw32", ctypes.c_int64),
                ("db", ctypes.c_void_p),
                ("act_below", ctypes.c_int32), ("accumulate_db", ctypes.c_int32)]

    @classmethod
    def make(cls, layer: Layer, pre=None, ldpre=0, act_below=0, dW32=None, lddw32=0, db=None, accumulate_db=0):
        return cls(layer, pre, ldpre, dW32, lddw32, db, act_below, accumulate_db)


_lib: Optional[ctypes.CDLL] = None


def library_path() -> str:
    return _LIB_PATH


def library() -> ctypes.CDLL:
    """Load libaxo.so (built in-tree by paper_2305_13525_amd/build.py).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is not built; run `python -m paper_2305_13525_amd.build` (needs hipcc). "
            "There is no fallback implementation.")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    PP = ctypes.POINTER(Problem)
    P64 = ctypes.POINTER(ctypes.c_int64)
    L.axo_version.restype = i32
    L.axo_status_string.argtypes = [i32]
    L.axo_status_string.restype = ctypes.c_char_p
    L.axo_shard_dims.argtypes = [PP, P64, P64, P64, P64, P64, P64]
    L.axo_shard_dims.restype = i32
    L.axo_workspace_bytes.argtypes = [PP, i32]
    L.axo_workspace_bytes.restype = sz
    L.axo_fc_route.argtypes = [PP, i32, i64, i64, i64, ctypes.POINTER(ctypes.c_int)]
    L.axo_fc_route.restype = i32
    L.axo_fc_fwd.argtypes = [PP, vp, i64, vp, i64, vp, i32, vp, i64, vp, sz, vp]
    L.axo_fc_fwd.restype = i32
    L.axo_fc_dgrad.argtypes = [PP, vp, i64, vp, i64, vp, i64, vp, sz, vp]
    L.axo_fc_dgrad.restype = i32
    L.axo_fc_wgrad.argtypes = [PP, vp, i64, vp, i64, vp, i64, vp, sz, vp]
    L.axo_fc_wgrad.restype = i32
    L.axo_layer_step_workspace_bytes.argtypes = [ctypes.POINTER(Layer), i32]
    L.axo_layer_step_workspace_bytes.restype = sz
    L.axo_layer_step.argtypes = [ctypes.POINTER(Layer), i32, vp, sz, vp]
    L.axo_layer_step.restype = i32
    L.axo_fc_dgrad_act.argtypes = [PP, vp, i64, vp, i64, vp, i64, i32, vp, i64, vp, sz, vp]
    L.axo_fc_dgrad_act.restype = i32
    L.axo_fc_wgrad_acc.argtypes = [PP, vp, i64, vp, i64, vp, i64, vp, sz, vp]
    L.axo_fc_wgrad_acc.restype = i32
    L.axo_bias_grad.argtypes = [PP, vp, i64, vp, i32, vp]
    L.axo_bias_grad.restype = i32
    L.axo_bias_grad_workspace_bytes.argtypes = [PP]
    L.axo_bias_grad_workspace_bytes.restype = sz
    L.axo_bias_grad_ws.argtypes = [PP, vp, i64, vp, i32, vp, sz, vp]
    L.axo_bias_grad_ws.restype = i32
    L.axo_bias_grad_static.argtypes = [PP, vp, i64, vp, i32, vp]
    L.axo_bias_grad_static.restype = i32
    L.axo_bias_grad_static_limit.restype = sz
    L.axo_layer_step_ext.argtypes = [ctypes.POINTER(LayerExt), i32, vp, sz, vp]
    L.axo_layer_step_ext.restype = i32
    L.axo_layer_step_ordered.argtypes = [ctypes.POINTER(Layer), i32, vp, sz, vp]
    L.axo_layer_step_ordered.restype = i32
    L.axo_layer_step_levels.argtypes = [ctypes.POINTER(Layer), i32, ctypes.POINTER(ctypes.c_int),
                                        ctypes.POINTER(ctypes.c_int)]
    L.axo_layer_step_levels.restype = i32
    _lib = L
    return L


def _check(rc: int, where: str, check: bool) -> int:
    if check and rc != 0:
        raise AxoError(rc, where)
    return rc


def axo_version() -> int:
    return int(library().axo_version())


def axo_status_string(status: int) -> str:
    return library().axo_status_string(int(status)).decode()


def axo_shard_dims(p: Optional[Problem], check: bool = True):
    """Returns (status, (M, Kl, Nl, row0, k0, n0))."""
    out = [ctypes.c_int64(0) for _ in range(6)]
    rc = library().axo_shard_dims(ctypes.byref(p) if p is not None else None, *[ctypes.byref(o) for o in out])
    _check(rc, "axo_shard_dims", check)
    return rc, tuple(int(o.value) for o in out)


def axo_workspace_bytes(p: Problem, op: int) -> int:
    return int(library().axo_workspace_bytes(ctypes.byref(p), int(op)))


def axo_fc_route(p: Problem, op: int, ld_a: int, ld_b: int, ld_out: int, check: bool = True) -> Tuple[int, int]:
    """(status, axo_route_t): which kernels the product takes for these leading dimensions."""
    r = ctypes.c_int(-1)
    rc = library().axo_fc_route(ctypes.byref(p) if p is not None else None, int(op), ld_a, ld_b, ld_out,
                                ctypes.byref(r))
    return _check(rc, "axo_fc_route", check), int(r.value)


def axo_fc_fwd(p: Problem, X: int, ldx: int, W: int, ldw: int, bias: Optional[int], epilogue: int, Y: int,
               ldy: int, ws: Optional[int] = None, ws_bytes: int = 0, stream: Optional[int] = None,
               check: bool = True) -> int:
    rc = library().axo_fc_fwd(ctypes.byref(p) if p is not None else None, X, ldx, W, ldw, bias, int(epilogue),
                              Y, ldy, ws, ws_bytes, stream)
    return _check(rc, "axo_fc_fwd", check)


def axo_fc_dgrad(p: Problem, dY: int, lddy: int, W: int, ldw: int, dX: int, lddx: int, ws: Optional[int] = None,
                 ws_bytes: int = 0, stream: Optional[int] = None, check: bool = True) -> int:
    rc = library().axo_fc_dgrad(ctypes.byref(p) if p is not None else None, dY, lddy, W, ldw, dX, lddx,
                                ws, ws_bytes, stream)
    return _check(rc, "axo_fc_dgrad", check)


def axo_fc_wgrad(p: Problem, X: int, ldx: int, dY: int, lddy: int, dW: int, lddw: int, ws: Optional[int] = None,
                 ws_bytes: int = 0, stream: Optional[int] = None, check: bool = True) -> int:
    rc = library().axo_fc_wgrad(ctypes.byref(p) if p is not None else None, X, ldx, dY, lddy, dW, lddw,
                                ws, ws_bytes, stream)
    return _check(rc, "axo_fc_wgrad", check)


def _layer_array(layers: Sequence[Layer]):
    arr = (Layer * max(1, len(layers)))()
    for i, l in enumerate(layers):
        arr[i] = l
    return arr


def axo_layer_step_workspace_bytes(layers: Sequence[Layer]) -> int:
    return int(library().axo_layer_step_workspace_bytes(_layer_array(layers), len(layers)))


def axo_layer_step(layers: Sequence[Layer], ws: Optional[int] = None, ws_bytes: int = 0,
                   stream: Optional[int] = None, check: bool = True) -> int:
    rc = library().axo_layer_step(_layer_array(layers), len(layers), ws, ws_bytes, stream)
    return _check(rc, "axo_layer_step", check)


def axo_layer_step_ext(layers: Sequence[LayerExt], ws: Optional[int] = None, ws_bytes: int = 0,
                       stream: Optional[int] = None, check: bool = True) -> int:
    arr = (LayerExt * max(1, len(layers)))()
    for i, l in enumerate(layers):
        arr[i] = l
    rc = library().axo_layer_step_ext(arr, len(layers), ws, ws_bytes, stream)
    return _check(rc, "axo_layer_step_ext", check)


def axo_layer_step_ordered(layers: Sequence[Layer], ws: Optional[int] = None, ws_bytes: int = 0,
                           stream: Optional[int] = None, check: bool = True) -> int:
    rc = library().axo_layer_step_ordered(_layer_array(layers), len(layers), ws, ws_bytes, stream)
    return _check(rc, "axo_layer_step_ordered", check)


def axo_layer_step_levels(layers: Sequence[Layer], check: bool = True) -> Tuple[int, int, list]:
    """(status, number of dependence levels, level of each of the 3 * len(layers) products)."""
    n = ctypes.c_int(0)
    lv = (ctypes.c_int * max(1, 3 * len(layers)))()
    rc = library().axo_layer_step_levels(_layer_array(layers), len(layers), ctypes.byref(n), lv)
    return _check(rc, "axo_layer_step_levels", check), int(n.value), list(lv)[:3 * len(layers)]


def axo_fc_dgrad_act(p: Problem, dY: int, lddy: int, W: int, ldw: int, pre: int, ldpre: int, act: int, dX: int,
                     lddx: int, ws: Optional[int] = None, ws_bytes: int = 0, stream: Optional[int] = None,
                     check: bool = True) -> int:
    rc = library().axo_fc_dgrad_act(ctypes.byref(p), dY, lddy, W, ldw, pre, ldpre, act, dX, lddx, ws, ws_bytes, stream)
    return _check(rc, "axo_fc_dgrad_act", check)


def axo_fc_wgrad_acc(p: Problem, X: int, ldx: int, dY: int, lddy: int, dW: int, lddw: int, ws: Optional[int] = None,
                     ws_bytes: int = 0, stream: Optional[int] = None, check: bool = True) -> int:
    rc = library().axo_fc_wgrad_acc(ctypes.byref(p), X, ldx, dY, lddy, dW, lddw, ws, ws_bytes, stream)
    return _check(rc, "axo_fc_wgrad_acc", check)


def axo_bias_grad(p: Problem, dY: int, lddy: int, db: int, accumulate: int = 0, stream: Optional[int] = None,
                  check: bool = True) -> int:
    rc = library().axo_bias_grad(ctypes.byref(p), dY, lddy, db, accumulate, stream)
    return _check(rc, "axo_bias_grad", check)


def axo_bias_grad_workspace_bytes(p: Problem) -> int:
    return int(library().axo_bias_grad_workspace_bytes(ctypes.byref(p)))


def axo_bias_grad_ws(p: Problem, dY: int, lddy: int, db: int, accumulate: int = 0, ws: Optional[int] = None,
                     ws_bytes: int = 0, stream: Optional[int] = None, check: bool = True) -> int:
    rc = library().axo_bias_grad_ws(ctypes.byref(p), dY, lddy, db, accumulate, ws, ws_bytes, stream)
    return _check(rc, "axo_bias_grad_ws", check)


def axo_bias_grad_static(p: Problem, dY: int, lddy: int, db: int, accumulate: int = 0, stream: Optional[int] = None,
                         check: bool = True) -> int:
    rc = library().axo_bias_grad_static(ctypes.byref(p), dY, lddy, db, accumulate, stream)
    return _check(rc, "axo_bias_grad_static", check)


def axo_bias_grad_static_limit() -> int:
    return int(library().axo_bias_grad_static_limit())
