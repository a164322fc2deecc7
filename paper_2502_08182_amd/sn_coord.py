"""ctypes binding of the bandwidth-coordinator entry points (include/sn_coord.h): the same
names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
from typing import Sequence, Tuple

from . import sn as _sn

EXPORTS = ("sn_coord_offloaded", "sn_coord_host_bytes", "sn_coord_rate", "sn_coord_adjust")


class sn_coord_instance(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_min", C.c_int32), ("n_max", C.c_int32), ("reserved", C.c_int32),
                ("mem_per_layer", C.c_uint64), ("iter_ns", C.c_int64)]


_ready = False


def _lib():
    global _ready
    L = _sn.lib()
    if not _ready:
        pi = C.POINTER(sn_coord_instance)
        L.sn_coord_offloaded.restype, L.sn_coord_offloaded.argtypes = C.c_int32, [pi, C.c_int32]
        L.sn_coord_host_bytes.restype, L.sn_coord_host_bytes.argtypes = C.c_uint64, [pi, C.c_int32]
        L.sn_coord_rate.restype, L.sn_coord_rate.argtypes = C.c_uint64, [pi, C.c_int32]
        L.sn_coord_adjust.restype = C.c_int
        L.sn_coord_adjust.argtypes = [pi, C.c_int32, C.c_uint64, C.POINTER(C.c_int32), C.POINTER(C.c_uint64),
                                      C.POINTER(C.c_uint64)]
        _ready = True
    return L


def make_instance(n_layers: int, mem_per_layer: int, iter_ns: int, n_min: int, n_max: int) -> sn_coord_instance:
    return sn_coord_instance(n_layers, n_min, n_max, 0, mem_per_layer, iter_ns)


def sn_coord_offloaded(inst: sn_coord_instance, N: int) -> int:
    return int(_lib().sn_coord_offloaded(C.byref(inst), N))


def sn_coord_host_bytes(inst: sn_coord_instance, N: int) -> int:
    return int(_lib().sn_coord_host_bytes(C.byref(inst), N))


def sn_coord_rate(inst: sn_coord_instance, N: int) -> int:
    return int(_lib().sn_coord_rate(C.byref(inst), N))


def sn_coord_adjust(instances: Sequence[sn_coord_instance], bandwidth_bytes_per_s: int) -> Tuple[Tuple[int, ...], int, int]:
    """Returns (intervals, total host bytes, total bytes/s); raises SnError(SN_E_INFEASIBLE) if none is valid."""
    n = len(instances)
    arr = (sn_coord_instance * n)(*instances)
    out = (C.c_int32 * n)()
    mem, rate = C.c_uint64(0), C.c_uint64(0)
    rc = _lib().sn_coord_adjust(arr, n, int(bandwidth_bytes_per_s), out, C.byref(mem), C.byref(rate))
    if rc != 0:
        raise _sn.SnError(rc, "sn_coord_adjust")
    return tuple(int(v) for v in out), int(mem.value), int(rate.value)
