"""ctypes binding of the per-kernel entry points (include/sn_kernels.h): same names,
argument marshalling only."""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import sn as _sn

EXPORTS = ("sn_k_tile_weights", "sn_k_norm", "sn_k_gemm", "sn_k_rope_append", "sn_k_attn_decode",
           "sn_k_attn_decode_append", "sn_k_attn_decode_append_planes", "sn_k_attn_decode_static",
           "sn_k_attn_prefill", "sn_k_cast_in", "sn_k_cast_out", "sn_k_copy", "sn_k_gemm_splitk", "sn_k_norm_fold", "sn_k_cast_out_fold", "sn_k_packed_offset")

EPI_STORE16, EPI_GELU16, EPI_RESID32, EPI_SWIGLU16 = 0, 1, 2, 3
PATH_SKINNY, PATH_TILE = 0, 1
SN_K_PREFILL_QTILE = 128    # query rows per prefill-attention tile (include/sn_kernels.h)

_ready = False


def _lib():
    global _ready
    L = _sn.lib()
    if not _ready:
        v, i32, u64 = C.c_void_p, C.c_int32, C.c_uint64
        sig = {
            "sn_k_tile_weights": [v, v, i32, i32, i32, i32, i32],
            "sn_k_norm": [i32, i32, v, v, v, v, i32, i32, C.c_float, v],
            "sn_k_gemm": [i32, i32, i32, v, v, v, v, i32, i32, i32, i32, v],
            "sn_k_packed_offset": [i32, i32, i32],
            "sn_k_rope_append": [i32, i32, v, v, v, v, v, v, v, v, i32, i32, i32, i32, i32, v],
            "sn_k_attn_decode": [i32, v, v, v, v, v, v, v, i32, i32, i32, i32, i32, i32, i32, v],
            "sn_k_attn_decode_static": [i32, v, v, v, v, v, v, i32, i32, i32, i32, i32, i32, i32, v],
            "sn_k_attn_decode_append": [i32, v, v, v, v, i32, v, v, v, v, v, i32, i32, i32, i32, i32, i32, i32, v],
            "sn_k_attn_decode_append_planes": [i32, v, i32, i32, v, v, v, i32, v, v, v, v, v, i32, i32, i32, i32, i32, i32, i32, v],
            "sn_k_attn_prefill": [i32, v, v, v, v, v, v, v, v, v, v, i32, i32, i32, i32, i32, v],
            "sn_k_cast_in": [i32, v, v, u64, v],
            "sn_k_cast_out": [i32, v, v, u64, v],
            "sn_k_copy": [v, v, u64, v],
            "sn_k_gemm_splitk": [i32, v, v, v, v, i32, i32, i32, i32, i32, v],
            "sn_k_norm_fold": [i32, i32, v, v, v, v, i32, i32, C.c_float, v, i32, v, i32, v],
            "sn_k_cast_out_fold": [i32, v, v, i32, i32, v, i32, v, v],
        }
        for name, args in sig.items():
            f = getattr(L, name)
            f.restype = (C.c_int64 if name == "sn_k_tile_weights" else
                         C.c_uint64 if name == "sn_k_packed_offset" else C.c_int)
            f.argtypes = args
        _ready = True
    return L


def _chk(rc):
    if rc != 0:
        raise _sn.SnError(rc, "kernel entry point rejected its arguments or the launch failed")


_p = _sn._ptr


def sn_k_tile_weights(src: np.ndarray, N: int, K: int, dst: np.ndarray = None, stride: int = 1, offset: int = 0,
                      bf16_to_f16: bool = False, return_bad: bool = False):
    src = np.ascontiguousarray(src, dtype=np.uint16)
    if dst is None:
        dst = np.zeros(N * K * stride, dtype=np.uint16)
    bad = _lib().sn_k_tile_weights(src.ctypes.data, dst.ctypes.data, N, K, stride, offset, int(bf16_to_f16))
    if bad < 0:
        _chk(int(bad))
    return (dst, int(bad)) if return_bad else dst


def sn_k_norm(dtype, is_ln, x32, gain, shift, out16, T, h, eps, stream=0):
    _chk(_lib().sn_k_norm(dtype, int(is_ln), _p(x32), _p(gain), _p(shift), _p(out16), T, h, eps, stream))


def sn_k_gemm(dtype, epilogue, path, W, X, bias, out, M, N, K, flags=0, stream=0):
    _chk(_lib().sn_k_gemm(dtype, epilogue, path, _p(W), _p(X), _p(bias), _p(out), M, N, K, flags, stream))


def sn_k_packed_offset(m, k, K) -> int:
    return int(_lib().sn_k_packed_offset(m, k, K))


def pack_rows(x: np.ndarray) -> np.ndarray:
    """Host helper (marshalling only): row-major [M][K] -> the row-tile packed layout."""
    M, K = x.shape
    Mp = (M + 15) // 16 * 16
    xp = np.zeros((Mp, K), dtype=x.dtype)
    xp[:M] = x
    return np.ascontiguousarray(xp.reshape(Mp // 16, 16, K // 32, 4, 8).transpose(0, 2, 3, 1, 4)).reshape(-1)


def unpack_rows(p: np.ndarray, M: int, K: int) -> np.ndarray:
    Mp = (M + 15) // 16 * 16
    return np.ascontiguousarray(p.reshape(Mp // 16, K // 32, 4, 16, 8).transpose(0, 3, 1, 2, 4)).reshape(Mp, K)[:M]


def sn_k_rope_append(dtype, kv_value_dtype, qkv16, tok_seq, tok_pos, kv_off, cap, kv, mirror, inv_freq, T, Hq, Hkv,
                     d, rope, stream=0):
    _chk(_lib().sn_k_rope_append(dtype, kv_value_dtype, _p(qkv16), _p(tok_seq), _p(tok_pos), _p(kv_off), _p(cap), _p(kv),
                                 _p(mirror), _p(inv_freq), T, Hq, Hkv, d, int(rope), stream))


def sn_k_attn_decode(dtype, qkv16, kv, len_before, kv_off, cap, out16, part, B, Hq, Hkv, d, S, max_len,
                     packed_out=0, stream=0):
    _chk(_lib().sn_k_attn_decode(dtype, _p(qkv16), _p(kv), _p(len_before), _p(kv_off), _p(cap), _p(out16),
                                 _p(part), B, Hq, Hkv, d, S, max_len, packed_out, stream))


SN_K_STATIC_SCRATCH_BYTES = 16 << 20    # include/sn_kernels.h


def sn_k_attn_decode_static(dtype, qkv16, kv, len_before, kv_off, cap, out16, B, Hq, Hkv, d, S, max_len,
                            packed_out=0, stream=0):
    rc = _lib().sn_k_attn_decode_static(dtype, _p(qkv16), _p(kv), _p(len_before), _p(kv_off), _p(cap), _p(out16),
                                        B, Hq, Hkv, d, S, max_len, packed_out, stream)
    if rc != 0:
        raise _sn.SnError(rc, _sn.sn_last_error(None))


def sn_k_attn_decode_append(dtype, qkv16, kv, mirror, inv_freq, rope, len_before, kv_off, cap, out16, part, B, Hq,
                            Hkv, d, S, max_len, packed_out=0, stream=0):
    _chk(_lib().sn_k_attn_decode_append(dtype, _p(qkv16), _p(kv), _p(mirror), _p(inv_freq), int(rope), _p(len_before),
                                        _p(kv_off), _p(cap), _p(out16), _p(part), B, Hq, Hkv, d, S, max_len,
                                        packed_out, stream))


def sn_k_attn_decode_append_planes(dtype, qkv_part, splits, plane_rows, kv, mirror, inv_freq, rope, len_before, kv_off,
                                   cap, out16, part, B, Hq, Hkv, d, S, max_len, packed_out=0, stream=0):
    _chk(_lib().sn_k_attn_decode_append_planes(dtype, _p(qkv_part), splits, plane_rows, _p(kv), _p(mirror), _p(inv_freq),
                                               int(rope), _p(len_before), _p(kv_off), _p(cap), _p(out16), _p(part),
                                               B, Hq, Hkv, d, S, max_len, packed_out, stream))


def sn_k_attn_prefill(dtype, qkv16, kv, len_before, n_new, tok_start, kv_off, cap, tile_seq, tile_q0, out16,
                      n_qtiles, Hq, Hkv, d, packed_out=0, stream=0):
    _chk(_lib().sn_k_attn_prefill(dtype, _p(qkv16), _p(kv), _p(len_before), _p(n_new), _p(tok_start), _p(kv_off),
                                  _p(cap), _p(tile_seq), _p(tile_q0), _p(out16), n_qtiles, Hq, Hkv, d, packed_out,
                                  stream))


def sn_k_cast_in(dtype, in16, x32, n, stream=0):
    _chk(_lib().sn_k_cast_in(dtype, _p(in16), _p(x32), n, stream))


def sn_k_cast_out(dtype, x32, out16, n, stream=0):
    _chk(_lib().sn_k_cast_out(dtype, _p(x32), _p(out16), n, stream))


def sn_k_copy(src, dst, nbytes, stream=0):
    _chk(_lib().sn_k_copy(_p(src), _p(dst), nbytes, stream))


def sn_k_gemm_splitk(dtype, W, X, bias, part, M, N, K, splits=0, flags=0, stream=0) -> int:
    rc = _lib().sn_k_gemm_splitk(dtype, _p(W), _p(X), _p(bias), _p(part), M, N, K, splits, flags, stream)
    if rc <= 0:
        _chk(rc if rc < 0 else -1)
    return rc


def sn_k_norm_fold(dtype, is_ln, x32, gain, shift, out16, T, h, eps, part, splits, bias, packed_out=0, stream=0):
    _chk(_lib().sn_k_norm_fold(dtype, int(is_ln), _p(x32), _p(gain), _p(shift), _p(out16), T, h, eps, _p(part), splits,
                               _p(bias), packed_out, stream))


def sn_k_cast_out_fold(dtype, x32, out16, T, h, part, splits, bias, stream=0):
    _chk(_lib().sn_k_cast_out_fold(dtype, _p(x32), _p(out16), T, h, _p(part), splits, _p(bias), stream))
