"""ctypes binding of the performance-record entry points (include/sn_record.h): the same
names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
from typing import Optional, Sequence

import numpy as np

from . import sn as _sn

SN_PHASE_DECODE, SN_PHASE_PREFILL = 0, 1
SN_SLO_ABS_NS, SN_SLO_REL_PERMILLE = 0, 1

EXPORTS = ("sn_record_create", "sn_record_destroy", "sn_record_layers", "sn_record_cells", "sn_record_put",
           "sn_record_profile", "sn_record_get", "sn_record_cell_interval", "sn_record_lookup", "sn_record_lookup_refined", "sn_record_table",
           "sn_record_save", "sn_record_load")

_ready = False


def _lib():
    global _ready
    L = _sn.lib()
    if not _ready:
        rec, ctx = C.c_void_p, C.c_void_p
        i32, i64 = C.c_int32, C.c_int64
        pi32, pi64 = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
        sig = {
            "sn_record_create": (C.c_int, [C.POINTER(rec), i32, i64]),
            "sn_record_destroy": (None, [rec]),
            "sn_record_layers": (i32, [rec]),
            "sn_record_cells": (i32, [rec]),
            "sn_record_put": (C.c_int, [rec, i32, i32, i32, pi64, pi64, i32]),
            "sn_record_profile": (C.c_int, [rec, ctx, i32, i32, i32, i32]),
            "sn_record_get": (C.c_int, [rec, i32, i32, i32, pi64, pi64, pi32]),
            "sn_record_cell_interval": (C.c_int, [rec, i32, i32, i32, i32, i64, pi32]),
            "sn_record_lookup": (C.c_int, [rec, i32, i32, i32, i32, i64, pi32]),
            "sn_record_lookup_refined": (C.c_int, [rec, i32, i32, i32, i32, i64, pi32]),
            "sn_record_table": (C.c_int, [rec, i32, i32, i64, pi32, i32, pi32, i32, pi32]),
            "sn_record_save": (C.c_int, [rec, C.c_char_p]),
            "sn_record_load": (C.c_int, [C.POINTER(rec), C.c_char_p]),
        }
        for name, (res, args) in sig.items():
            f = getattr(L, name)
            f.restype = res
            f.argtypes = args
        _ready = True
    return L


def _chk(rc: int, what: str):
    if rc != 0:
        raise _sn.SnError(rc, what)


def _i64(a):
    arr = np.ascontiguousarray(a, dtype=np.int64)
    return arr, arr.ctypes.data_as(C.POINTER(C.c_int64))


def _i32(a):
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(C.POINTER(C.c_int32))


def sn_record_create(n_layers: int, slo_step_ns: int = 0):
    rec = C.c_void_p()
    _chk(_lib().sn_record_create(C.byref(rec), n_layers, slo_step_ns), "sn_record_create")
    return rec


def sn_record_destroy(rec) -> None:
    _lib().sn_record_destroy(rec)


def sn_record_layers(rec) -> int:
    return int(_lib().sn_record_layers(rec))


def sn_record_cells(rec) -> int:
    return int(_lib().sn_record_cells(rec))


def sn_record_put(rec, phase: int, batch: int, seq: int, tc_ns: Sequence[int], tx_ns: Sequence[int], n_max: int) -> None:
    L = sn_record_layers(rec)
    if len(tc_ns) != L or len(tx_ns) != L:
        raise ValueError("tc_ns and tx_ns need one entry per layer")
    a, pa = _i64(tc_ns)
    b, pb = _i64(tx_ns)
    _chk(_lib().sn_record_put(rec, phase, batch, seq, pa, pb, n_max), "sn_record_put")


def sn_record_profile(rec, ctx, phase: int, batch: int, seq: int, reps: int = 3) -> None:
    rc = _lib().sn_record_profile(rec, ctx, phase, batch, seq, reps)
    if rc != 0:
        msg = _sn.lib().sn_last_error(ctx)
        raise _sn.SnError(rc, msg.decode() if msg else "sn_record_profile")


def sn_record_get(rec, phase: int, batch: int, seq: int):
    """Returns (tc_ns, tx_ns, n_max) of a stored cell."""
    L = sn_record_layers(rec)
    tc, ptc = _i64(np.zeros(L, dtype=np.int64))
    tx, ptx = _i64(np.zeros(L, dtype=np.int64))
    n = C.c_int32(0)
    _chk(_lib().sn_record_get(rec, phase, batch, seq, ptc, ptx, C.byref(n)), "sn_record_get")
    return tc, tx, int(n.value)


def sn_record_cell_interval(rec, phase: int, batch: int, seq: int, slo_kind: int, slo_value: int) -> int:
    n = C.c_int32(0)
    _chk(_lib().sn_record_cell_interval(rec, phase, batch, seq, slo_kind, int(slo_value), C.byref(n)),
         "sn_record_cell_interval")
    return int(n.value)


def sn_record_lookup(rec, phase: int, batch: int, seq: int, slo_kind: int, slo_value: int) -> int:
    n = C.c_int32(0)
    _chk(_lib().sn_record_lookup(rec, phase, batch, seq, slo_kind, int(slo_value), C.byref(n)), "sn_record_lookup")
    return int(n.value)


def sn_record_lookup_refined(rec, phase: int, batch: int, seq: int, slo_kind: int, slo_value: int) -> int:
    n = C.c_int32(0)
    _chk(_lib().sn_record_lookup_refined(rec, phase, batch, seq, slo_kind, int(slo_value), C.byref(n)), "sn_record_lookup_refined")
    return int(n.value)


def sn_record_table(rec, phase: int, slo_kind: int, slo_value: int, batches: Sequence[int], seqs: Sequence[int]):
    b, pb = _i32(batches)
    s, ps = _i32(seqs)
    out, po = _i32(np.zeros(len(b) * len(s), dtype=np.int32))
    _chk(_lib().sn_record_table(rec, phase, slo_kind, int(slo_value), pb, len(b), ps, len(s), po), "sn_record_table")
    return out.reshape(len(b), len(s))


def sn_record_save(rec, path: str) -> None:
    _chk(_lib().sn_record_save(rec, path.encode()), f"sn_record_save({path})")


def sn_record_load(path: str):
    rec = C.c_void_p()
    _chk(_lib().sn_record_load(C.byref(rec), path.encode()), f"sn_record_load({path})")
    return rec
