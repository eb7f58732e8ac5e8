"""ctypes binding of the host-only communication-model functions of libaxo.so (include/axo_comm.h):
argument marshalling only, same names as the C functions."""
from __future__ import annotations

import ctypes
from typing import List, Optional, Sequence, Tuple

from .binding import AxoError, library


class CommConfig(ctypes.Structure):
    _fields_ = [("Gx", ctypes.c_int32), ("Gy", ctypes.c_int32), ("Gz", ctypes.c_int32), ("Gdata", ctypes.c_int32)]

    def as_tuple(self) -> Tuple[int, int, int, int]:
        return (self.Gx, self.Gy, self.Gz, self.Gdata)


class CommNet(ctypes.Structure):
    _fields_ = [("beta_intra", ctypes.c_double), ("beta_inter", ctypes.c_double), ("G_node", ctypes.c_int32),
                ("placement_aware", ctypes.c_int32)]


class CommLayer(ctypes.Structure):
    _fields_ = [("k", ctypes.c_int64), ("n", ctypes.c_int64), ("transposed", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class CommTerms(ctypes.Structure):
    _fields_ = [("ag_z", ctypes.c_double), ("rs_z", ctypes.c_double), ("ar_fwd", ctypes.c_double),
                ("ar_bwd", ctypes.c_double), ("ar_data", ctypes.c_double), ("total", ctypes.c_double)]


_ready = False


def _lib():
    global _ready
    L = library()
    if not _ready:
        d, i32, i64 = ctypes.c_double, ctypes.c_int32, ctypes.c_int64
        PC, PN, PL, PT = (ctypes.POINTER(CommConfig), ctypes.POINTER(CommNet), ctypes.POINTER(CommLayer),
                          ctypes.POINTER(CommTerms))
        for name in ("axo_comm_ring_all_gather", "axo_comm_ring_reduce_scatter", "axo_comm_ring_all_reduce"):
            getattr(L, name).argtypes = [i32, d, d]
            getattr(L, name).restype = d
        L.axo_comm_net_mi355x.argtypes = [PN]
        L.axo_comm_bandwidths.argtypes = [PC, PN, ctypes.POINTER(d)]
        L.axo_comm_layer_time.argtypes = [PC, PN, PL, i64, d, PT]
        L.axo_comm_model_time.argtypes = [PC, PN, PL, i32, i64, d, ctypes.POINTER(d), PT]
        L.axo_comm_rank_configs.argtypes = [i32, PN, PL, i32, i64, d, PC, ctypes.POINTER(d), i32, ctypes.POINTER(i32)]
        L.axo_comm_rank_to_coord.argtypes = [PC, i64, ctypes.POINTER(i32)]
        L.axo_comm_coord_to_rank.argtypes = [PC, ctypes.POINTER(i32), ctypes.POINTER(i64)]
        for name in ("axo_comm_net_mi355x", "axo_comm_bandwidths", "axo_comm_layer_time", "axo_comm_model_time",
                     "axo_comm_rank_configs", "axo_comm_rank_to_coord", "axo_comm_coord_to_rank"):
            getattr(L, name).restype = ctypes.c_int
        _ready = True
    return L


def _check(rc: int, where: str, check: bool) -> int:
    if rc != 0 and check:
        raise AxoError(rc, where)
    return rc


def _layers(layers: Sequence[CommLayer]):
    return (CommLayer * max(len(layers), 1))(*layers)


def axo_comm_ring_all_gather(G: int, nbytes: float, beta: float) -> float:
    return float(_lib().axo_comm_ring_all_gather(G, nbytes, beta))


def axo_comm_ring_reduce_scatter(G: int, nbytes: float, beta: float) -> float:
    return float(_lib().axo_comm_ring_reduce_scatter(G, nbytes, beta))


def axo_comm_ring_all_reduce(G: int, nbytes: float, beta: float) -> float:
    return float(_lib().axo_comm_ring_all_reduce(G, nbytes, beta))


def axo_comm_net_mi355x() -> CommNet:
    net = CommNet()
    _check(_lib().axo_comm_net_mi355x(ctypes.byref(net)), "axo_comm_net_mi355x", True)
    return net


def axo_comm_bandwidths(cfg: CommConfig, net: CommNet, check: bool = True):
    beta = (ctypes.c_double * 4)()
    rc = _check(_lib().axo_comm_bandwidths(ctypes.byref(cfg), ctypes.byref(net), beta), "axo_comm_bandwidths", check)
    return rc, tuple(beta)


def axo_comm_layer_time(cfg: CommConfig, net: CommNet, layer: CommLayer, m_rows: int, bytes_per_element: float,
                        check: bool = True):
    t = CommTerms()
    rc = _check(_lib().axo_comm_layer_time(ctypes.byref(cfg), ctypes.byref(net), ctypes.byref(layer), m_rows,
                                           bytes_per_element, ctypes.byref(t)), "axo_comm_layer_time", check)
    return rc, t


def axo_comm_model_time(cfg: CommConfig, net: CommNet, layers: Sequence[CommLayer], batch_rows: int,
                        bytes_per_element: float, check: bool = True):
    total, t = ctypes.c_double(0.0), CommTerms()
    rc = _check(_lib().axo_comm_model_time(ctypes.byref(cfg), ctypes.byref(net), _layers(layers), len(layers),
                                           batch_rows, bytes_per_element, ctypes.byref(total), ctypes.byref(t)),
                "axo_comm_model_time", check)
    return rc, total.value, t


def axo_comm_rank_configs(n_gpus: int, net: CommNet, layers: Sequence[CommLayer], batch_rows: int,
                          bytes_per_element: float, max_out: int = 1 << 16, check: bool = True):
    """Returns (status, [(Gx, Gy, Gz, Gdata), ...], [seconds, ...], n_found)."""
    cfgs = (CommConfig * max(max_out, 1))()
    times = (ctypes.c_double * max(max_out, 1))()
    n = ctypes.c_int32(0)
    rc = _check(_lib().axo_comm_rank_configs(n_gpus, ctypes.byref(net), _layers(layers), len(layers), batch_rows,
                                             bytes_per_element, cfgs, times, max_out, ctypes.byref(n)),
                "axo_comm_rank_configs", check)
    k = min(n.value, max_out) if rc == 0 else 0
    return rc, [cfgs[i].as_tuple() for i in range(k)], [times[i] for i in range(k)], n.value


def axo_comm_rank_to_coord(cfg: CommConfig, rank: int, check: bool = True):
    c = (ctypes.c_int32 * 4)()
    rc = _check(_lib().axo_comm_rank_to_coord(ctypes.byref(cfg), rank, c), "axo_comm_rank_to_coord", check)
    return rc, tuple(c)


def axo_comm_coord_to_rank(cfg: CommConfig, coord: Sequence[int], check: bool = True):
    c = (ctypes.c_int32 * 4)(*coord)
    r = ctypes.c_int64(-1)
    rc = _check(_lib().axo_comm_coord_to_rank(ctypes.byref(cfg), c, ctypes.byref(r)), "axo_comm_coord_to_rank", check)
    return rc, r.value
