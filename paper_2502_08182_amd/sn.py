"""ctypes binding of libsn.so: the same names as include/sn.h, argument marshalling only.

Every step of the path runs inside the library's HIP kernels; this module never
computes.  If the library has not been built it raises -- there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libsn.so")

SN_F16, SN_BF16 = 0, 1
SN_ACT_GELU, SN_ACT_SWIGLU = 0, 1
SN_NORM_LN, SN_NORM_RMS = 0, 1
SN_SCHED_PAPER, SN_SCHED_EAGER, SN_SCHED_CONTINUOUS = 0, 1, 2
SN_OFFLOAD_STATE, SN_OFFLOAD_WEIGHTS, SN_OFFLOAD_KV = 0, 1, 2
SN_OK, SN_E_INVAL, SN_E_STATE, SN_E_BUDGET, SN_E_INFEASIBLE, SN_E_NOMEM, SN_E_HIP = 0, -1, -2, -3, -4, -5, -6
SN_DEBUG_POISON_SLOT, SN_DEBUG_DELAY_H2D, SN_DEBUG_DELAY_COMPUTE, SN_DEBUG_DELAY_D2H = 1, 2, 4, 8
SN_K_NAMES = ("norm", "qkv", "rope_append", "attn", "oproj", "ffn_up", "ffn_down", "other")
ERROR_NAMES = {-1: "SN_E_INVAL", -2: "SN_E_STATE", -3: "SN_E_BUDGET", -4: "SN_E_INFEASIBLE",
               -5: "SN_E_NOMEM", -6: "SN_E_HIP"}

EXPORTS = (
    "sn_init", "sn_destroy", "sn_last_error", "sn_layers", "sn_layer_blob_bytes", "sn_set_layer_weights", "sn_place",
    "sn_set_budget_enforce", "sn_resident_bytes", "sn_max_interval", "sn_max_tokens", "sn_placement", "sn_kv_reset", "sn_step",
    "sn_read_hidden_f32",
    "sn_set_timing", "sn_set_kernel_timing_class", "sn_time_kernel_class", "sn_get_stats", "sn_get_layer_times", "sn_profile_layers", "sn_timeline",
    "sn_pick_interval_from_times", "sn_pick_interval", "sn_paper_rule",
    "sn_set_schedule", "sn_placement_sched", "sn_timeline_sched", "sn_pick_interval_from_times_sched", "sn_refine_interval_from_times", "sn_refine_interval",
    "sn_set_offload_part", "sn_offload_part", "sn_max_tokens_part", "sn_resident_bytes_part",
    "sn_kv_truncate", "sn_set_debug",
)


class sn_model_shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn",
                                          "act", "norm", "rope", "has_bias", "dtype")] + \
               [("norm_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("max_batch", "max_seq", "max_tokens")]


class sn_batch(C.Structure):
    _fields_ = [("batch", C.c_int32), ("is_prefill", C.c_int32), ("n_new", C.POINTER(C.c_int32)),
                ("hidden_in", C.c_void_p)]


class sn_kv(C.Structure):
    _fields_ = [("len", C.POINTER(C.c_int32))]


class sn_step_stats(C.Structure):
    _fields_ = [("iter_ns", C.c_int64), ("stall_ns", C.c_int64), ("h2d_ns", C.c_int64), ("h2d_bytes", C.c_int64),
                ("d2h_ns", C.c_int64), ("d2h_bytes", C.c_int64), ("hidden_fraction", C.c_double),
                ("interval", C.c_int32), ("n_offloaded", C.c_int32), ("resident_bytes", C.c_uint64),
                ("kernel_ns", C.c_int64 * 8), ("kernel_calls", C.c_int32 * 8), ("n_preissued", C.c_int32),
                ("nonfinite", C.c_int32)]

    def as_dict(self) -> dict:
        d = {n: getattr(self, n) for n, _ in self._fields_ if n not in ("kernel_ns", "kernel_calls")}
        d["kernel_ns"] = {SN_K_NAMES[i]: self.kernel_ns[i] for i in range(8)}
        d["kernel_calls"] = {SN_K_NAMES[i]: self.kernel_calls[i] for i in range(8)}
        return d


class SnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{ERROR_NAMES.get(code, code)}: {msg}")
        self.code = code


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """Load libsn.so (built by paper_2502_08182_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2502_08182_amd.build` "
                           "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    ctx = C.c_void_p
    i32, i64, u64 = C.c_int32, C.c_int64, C.c_uint64
    pi32, pi64 = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    sig = {
        "sn_init": (C.c_int, [C.POINTER(ctx), C.POINTER(sn_model_shape), u64, C.c_void_p]),
        "sn_destroy": (None, [ctx]),
        "sn_last_error": (C.c_char_p, [ctx]),
        "sn_layers": (i32, [ctx]),
        "sn_layer_blob_bytes": (u64, [C.POINTER(sn_model_shape)]),
        "sn_set_layer_weights": (C.c_int, [ctx, i32, C.c_void_p, u64]),
        "sn_place": (C.c_int, [ctx, i32]),
        "sn_set_budget_enforce": (C.c_int, [ctx, i32]),
        "sn_resident_bytes": (u64, [ctx, i32]),
        "sn_max_interval": (i32, [ctx]),
        "sn_max_tokens": (u64, [i32, i32, u64, u64, u64, u64]),
        "sn_max_tokens_part": (u64, [i32, i32, u64, u64, u64, u64, i32]),
        "sn_resident_bytes_part": (u64, [i32, i32, u64, u64, u64, i32]),
        "sn_set_offload_part": (C.c_int, [ctx, i32]),
        "sn_offload_part": (i32, [ctx]),
        "sn_placement": (C.c_int, [i32, i32, C.POINTER(C.c_uint8), pi32]),
        "sn_kv_reset": (C.c_int, [ctx, i32, pi32]),
        "sn_kv_truncate": (C.c_int, [ctx, i32, pi32]),
        "sn_set_debug": (C.c_int, [ctx, i32, i32]),
        "sn_step": (C.c_int, [ctx, C.POINTER(sn_batch), C.POINTER(sn_kv), C.c_void_p]),
        "sn_read_hidden_f32": (C.c_int, [ctx, C.c_void_p, u64]),
        "sn_set_timing": (C.c_int, [ctx, i32]),
        "sn_set_kernel_timing_class": (C.c_int, [ctx, i32]),
        "sn_time_kernel_class": (C.c_int, [ctx, i32, i32, i32, pi64, pi32]),
        "sn_get_stats": (C.c_int, [ctx, C.POINTER(sn_step_stats)]),
        "sn_get_layer_times": (C.c_int, [ctx, pi64, pi64, pi64]),
        "sn_profile_layers": (C.c_int, [ctx, i32, i32, i32, i32, pi64, pi64]),
        "sn_timeline": (C.c_int, [i32, pi64, pi64, i32, pi64, pi64]),
        "sn_pick_interval_from_times": (C.c_int, [i32, pi64, pi64, i64, i32, pi32]),
        "sn_pick_interval": (C.c_int, [ctx, C.c_double, pi32]),
        "sn_refine_interval": (C.c_int, [ctx, i32, pi32]),
        "sn_paper_rule": (i32, [i32, i64, i64]),
        "sn_set_schedule": (C.c_int, [ctx, i32]),
        "sn_placement_sched": (C.c_int, [i32, i32, i32, C.POINTER(C.c_uint8), pi32]),
        "sn_timeline_sched": (C.c_int, [i32, pi64, pi64, i32, i32, pi64, pi64]),
        "sn_pick_interval_from_times_sched": (C.c_int, [i32, pi64, pi64, i64, i32, i32, pi32]),
        "sn_refine_interval_from_times": (C.c_int, [i32, pi64, pi64, i32, i32, pi32]),
    }
    for name, (res, args) in sig.items():
        f = getattr(L, name)
        f.restype = res
        f.argtypes = args
    _lib = L
    return L


def _check(rc: int, ctx=None):
    if rc != SN_OK:
        msg = lib().sn_last_error(ctx)
        raise SnError(rc, msg.decode() if msg else "")


def _ptr(x) -> int:
    """Device or host address of a torch tensor / numpy array / int."""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    if isinstance(x, np.ndarray):
        return int(x.ctypes.data)
    raise TypeError(type(x))


def _i64(a: Sequence[int]):
    arr = np.ascontiguousarray(a, dtype=np.int64)
    return arr, arr.ctypes.data_as(C.POINTER(C.c_int64))


def make_shape(ms, max_batch: int, max_seq: int, max_tokens: int = 0) -> sn_model_shape:
    """sn_model_shape from a synth.ModelShape-like object (attribute access)."""
    return sn_model_shape(
        n_layers=ms.n_layers, hidden=ms.hidden, n_q_heads=ms.n_q_heads, n_kv_heads=ms.n_kv_heads,
        head_dim=ms.head_dim, ffn=ms.ffn, act=SN_ACT_SWIGLU if ms.act == "swiglu" else SN_ACT_GELU,
        norm=SN_NORM_RMS if ms.norm == "rms" else SN_NORM_LN, rope=int(ms.rope), has_bias=int(ms.has_bias),
        dtype=SN_BF16 if ms.dtype == "bf16" else SN_F16, norm_eps=ms.norm_eps, rope_theta=ms.rope_theta,
        max_batch=max_batch, max_seq=max_seq, max_tokens=max_tokens)


# ---- the calls, same names as the header ------------------------------------------

def sn_init(shape: sn_model_shape, hbm_budget_bytes: int = 0, hip_compute_stream: int = 0) -> C.c_void_p:
    ctx = C.c_void_p()
    _check(lib().sn_init(C.byref(ctx), C.byref(shape), int(hbm_budget_bytes), C.c_void_p(hip_compute_stream)))
    return ctx


def sn_destroy(ctx) -> None:
    lib().sn_destroy(ctx)


def sn_last_error(ctx=None) -> str:
    m = lib().sn_last_error(ctx)
    return m.decode() if m else ""


def sn_layer_blob_bytes(shape: sn_model_shape) -> int:
    return int(lib().sn_layer_blob_bytes(C.byref(shape)))


def sn_set_layer_weights(ctx, layer: int, host_blob: np.ndarray) -> None:
    blob = np.ascontiguousarray(host_blob).view(np.uint8).reshape(-1)
    _check(lib().sn_set_layer_weights(ctx, layer, C.c_void_p(blob.ctypes.data), blob.size), ctx)


def sn_place(ctx, N: int) -> None:
    _check(lib().sn_place(ctx, N), ctx)


def sn_set_budget_enforce(ctx, on: bool) -> None:
    _check(lib().sn_set_budget_enforce(ctx, int(on)), ctx)


def sn_resident_bytes(ctx, N: int) -> int:
    return int(lib().sn_resident_bytes(ctx, N))


def sn_max_interval(ctx) -> int:
    return int(lib().sn_max_interval(ctx))


def sn_max_tokens(L: int, N: int, weight_bytes: int, kv_token_bytes: int, fixed_bytes: int, budget: int) -> int:
    return int(lib().sn_max_tokens(L, N, weight_bytes, kv_token_bytes, fixed_bytes, budget))


def sn_max_tokens_part(L: int, N: int, weight_bytes: int, kv_token_bytes: int, fixed_bytes: int, budget: int, what: int) -> int:
    return int(lib().sn_max_tokens_part(L, N, weight_bytes, kv_token_bytes, fixed_bytes, budget, what))


def sn_resident_bytes_part(L: int, N: int, weight_bytes: int, kv_bytes: int, fixed_bytes: int, what: int) -> int:
    return int(lib().sn_resident_bytes_part(L, N, weight_bytes, kv_bytes, fixed_bytes, what))


def sn_set_offload_part(ctx, what: int) -> None:
    _check(lib().sn_set_offload_part(ctx, what), ctx)


def sn_offload_part(ctx) -> int:
    return int(lib().sn_offload_part(ctx))


def sn_layers(ctx) -> int:
    return int(lib().sn_layers(ctx))


def sn_placement(L: int, N: int):
    off = np.zeros(L, dtype=np.uint8)
    trig = np.zeros(L, dtype=np.int32)
    _check(lib().sn_placement(L, N, off.ctypes.data_as(C.POINTER(C.c_uint8)),
                              trig.ctypes.data_as(C.POINTER(C.c_int32))))
    return off, trig


def sn_placement_sched(L: int, N: int, schedule: int):
    off = np.zeros(L, dtype=np.uint8)
    trig = np.zeros(L, dtype=np.int32)
    _check(lib().sn_placement_sched(L, N, schedule, off.ctypes.data_as(C.POINTER(C.c_uint8)),
                                    trig.ctypes.data_as(C.POINTER(C.c_int32))))
    return off, trig


def sn_set_schedule(ctx, schedule: int) -> None:
    _check(lib().sn_set_schedule(ctx, schedule), ctx)


def sn_kv_reset(ctx, capacity: Sequence[int]) -> None:
    cap = np.ascontiguousarray(capacity, dtype=np.int32)
    _check(lib().sn_kv_reset(ctx, cap.size, cap.ctypes.data_as(C.POINTER(C.c_int32))), ctx)


def sn_kv_truncate(ctx, length: Sequence[int]) -> None:
    ln = np.ascontiguousarray(length, dtype=np.int32)
    _check(lib().sn_kv_truncate(ctx, ln.size, ln.ctypes.data_as(C.POINTER(C.c_int32))), ctx)


def sn_set_debug(ctx, flags: int, delay_us: int = 0) -> None:
    _check(lib().sn_set_debug(ctx, int(flags), int(delay_us)), ctx)


def sn_step(ctx, n_new: Sequence[int], is_prefill: bool, hidden_in, kv_len: np.ndarray, hidden_out) -> None:
    """kv_len: int32 numpy array [batch], advanced in place by the library."""
    nn = np.ascontiguousarray(n_new, dtype=np.int32)
    assert kv_len.dtype == np.int32 and kv_len.flags["C_CONTIGUOUS"]
    b = sn_batch(batch=nn.size, is_prefill=int(is_prefill), n_new=nn.ctypes.data_as(C.POINTER(C.c_int32)),
                 hidden_in=C.c_void_p(_ptr(hidden_in)))
    kv = sn_kv(len=kv_len.ctypes.data_as(C.POINTER(C.c_int32)))
    _check(lib().sn_step(ctx, C.byref(b), C.byref(kv), C.c_void_p(_ptr(hidden_out))), ctx)


def sn_read_hidden_f32(ctx, dst, dst_bytes: int) -> None:
    _check(lib().sn_read_hidden_f32(ctx, C.c_void_p(_ptr(dst)), int(dst_bytes)), ctx)


def sn_set_timing(ctx, level: int) -> None:
    _check(lib().sn_set_timing(ctx, level), ctx)


def sn_set_kernel_timing_class(ctx, kernel_class: int) -> None:
    _check(lib().sn_set_kernel_timing_class(ctx, kernel_class), ctx)


def sn_time_kernel_class(ctx, kernel_class: int, batch: int, reps: int = 1):
    """Returns (total_ns, launches)."""
    ns, n = C.c_int64(), C.c_int32()
    _check(lib().sn_time_kernel_class(ctx, kernel_class, batch, reps, C.byref(ns), C.byref(n)), ctx)
    return ns.value, n.value


def sn_get_stats(ctx) -> sn_step_stats:
    st = sn_step_stats()
    _check(lib().sn_get_stats(ctx, C.byref(st)), ctx)
    return st


def sn_get_layer_times(ctx, L: int):
    a = [np.zeros(L, dtype=np.int64) for _ in range(3)]
    _check(lib().sn_get_layer_times(ctx, *[x.ctypes.data_as(C.POINTER(C.c_int64)) for x in a]), ctx)
    return tuple(a)


def sn_profile_layers(ctx, L: int, is_prefill: bool, batch: int, seq: int, reps: int = 3):
    tc = np.zeros(L, dtype=np.int64)
    tx = np.zeros(L, dtype=np.int64)
    _check(lib().sn_profile_layers(ctx, int(is_prefill), batch, seq, reps,
                                   tc.ctypes.data_as(C.POINTER(C.c_int64)),
                                   tx.ctypes.data_as(C.POINTER(C.c_int64))), ctx)
    return tc, tx


def sn_timeline(tc: Sequence[int], tx: Sequence[int], N: int):
    a, pa = _i64(tc)
    b, pb = _i64(tx)
    it, st = C.c_int64(), C.c_int64()
    _check(lib().sn_timeline(a.size, pa, pb, N, C.byref(it), C.byref(st)))
    return it.value, st.value


def sn_timeline_sched(tc: Sequence[int], tx: Sequence[int], N: int, schedule: int):
    a, pa = _i64(tc)
    b, pb = _i64(tx)
    it, st = C.c_int64(), C.c_int64()
    _check(lib().sn_timeline_sched(a.size, pa, pb, N, schedule, C.byref(it), C.byref(st)))
    return it.value, st.value


def sn_pick_interval_from_times_sched(tc: Sequence[int], tx: Sequence[int], slo_ns: int, n_max: int, schedule: int) -> int:
    a, pa = _i64(tc)
    b, pb = _i64(tx)
    out = C.c_int32()
    _check(lib().sn_pick_interval_from_times_sched(a.size, pa, pb, int(slo_ns), int(n_max), schedule, C.byref(out)))
    return out.value


def sn_refine_interval_from_times(tc: Sequence[int], tx: Sequence[int], N: int, schedule: int = 0) -> int:
    a, pa = _i64(tc)
    b, pb = _i64(tx)
    out = C.c_int32()
    _check(lib().sn_refine_interval_from_times(a.size, pa, pb, int(N), schedule, C.byref(out)))
    return out.value


def sn_pick_interval_from_times(tc: Sequence[int], tx: Sequence[int], slo_ns: int, n_max: int) -> int:
    a, pa = _i64(tc)
    b, pb = _i64(tx)
    out = C.c_int32()
    _check(lib().sn_pick_interval_from_times(a.size, pa, pb, int(slo_ns), int(n_max), C.byref(out)))
    return out.value


def sn_pick_interval(ctx, slo_ms: float) -> int:
    out = C.c_int32()
    _check(lib().sn_pick_interval(ctx, float(slo_ms), C.byref(out)), ctx)
    return out.value


def sn_refine_interval(ctx, N: int) -> int:
    out = C.c_int32()
    _check(lib().sn_refine_interval(ctx, int(N), C.byref(out)), ctx)
    return out.value


def sn_paper_rule(L: int, t_trans_ns: int, slo_ns: int) -> int:
    return int(lib().sn_paper_rule(L, int(t_trans_ns), int(slo_ns)))
