// C ABI of the individual layer kernels (include/sn_kernels.h): argument checks, then
// the same launchers sn_step uses.
#include <hip/hip_runtime.h>

#include "../../include/sn.h"
#include "../../include/sn_kernels.h"
#include "kernels.h"
#include "layout.h"

using namespace sn;

static int rc_of(hipError_t e) { return e == hipSuccess ? SN_OK : (e == hipErrorInvalidValue ? SN_E_INVAL : SN_E_HIP); }
static bool bad_dtype(int d) { return d != SN_F16 && d != SN_BF16; }

extern "C" uint64_t sn_k_packed_offset(int32_t m, int32_t k, int32_t K) {
  const int KB = K / 32;
  return ((((uint64_t)(m >> 4) * KB + (k >> 5)) * 64) + (m & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}

extern "C" int64_t sn_k_tile_weights(const void* src, void* dst, int32_t N, int32_t K, int32_t stride, int32_t offset,
                                     int32_t bf16_to_f16) {
  if (!src || !dst || N < 16 || K < 32 || N % 16 || K % 32 || stride < 1 || offset < 0 || offset >= stride)
    return SN_E_INVAL;
  return (int64_t)tile_matrix(static_cast<uint16_t*>(dst), static_cast<const uint16_t*>(src), N, K, stride, offset,
                              bf16_to_f16 != 0);
}

extern "C" int sn_k_norm(int32_t dtype, int32_t is_ln, const void* x32, const void* gain, const void* shift,
                         void* out16, int32_t T, int32_t h, float eps, void* stream) {
  if (bad_dtype(dtype) || !x32 || !gain || !out16 || T < 0 || h < 1 || (is_ln && !shift)) return SN_E_INVAL;
  return rc_of(launch_norm(dtype, is_ln, (const float*)x32, gain, shift, out16, T, h, eps, (hipStream_t)stream));
}

extern "C" int sn_k_gemm(int32_t dtype, int32_t epi, int32_t path, const void* W, const void* X, const void* bias,
                         void* out, int32_t M, int32_t N, int32_t K, int32_t flags, void* stream) {
  if (bad_dtype(dtype) || !W || !X || !out || M < 0 || N < 16 || K < 32 || epi < 0 || epi > 3 || flags < 0 || flags > 3)
    return SN_E_INVAL;
  if (path == 0) return rc_of(launch_gemm_skinny(dtype, epi, W, X, bias, out, M, N, K, (hipStream_t)stream, 1, flags));
  if (path == 1) return rc_of(launch_gemm_tile(dtype, epi, W, X, bias, out, M, N, K, (hipStream_t)stream, flags));
  return SN_E_INVAL;
}

extern "C" int sn_k_rope_append(int32_t dtype, int32_t kv_value_dtype, void* qkv16, const int32_t* tok_seq, const int32_t* tok_pos,
                                const int32_t* kv_off, const int32_t* cap, void* kv, void* mirror,
                                const float* inv_freq, int32_t T, int32_t Hq, int32_t Hkv, int32_t d, int32_t rope,
                                void* stream) {
  if (bad_dtype(dtype) || bad_dtype(kv_value_dtype) || (dtype == SN_BF16 && kv_value_dtype == SN_F16) || !qkv16 || !tok_seq || !tok_pos || !kv_off || !cap || !kv || (rope && !inv_freq) ||
      T < 0 || Hq < 1 || Hkv < 1 || (d != 64 && d != 128))
    return SN_E_INVAL;
  StepIndex ix{};
  ix.tok_seq = tok_seq;
  ix.tok_pos = tok_pos;
  ix.kv_off = kv_off;
  ix.cap = cap;
  return rc_of(launch_rope_append(dtype, kv_value_dtype, qkv16, ix, kv, mirror, inv_freq, T, Hq, Hkv, d, rope, (hipStream_t)stream));
}

extern "C" int sn_k_attn_decode(int32_t dtype, const void* qkv16, const void* kv, const int32_t* len_before,
                                const int32_t* kv_off, const int32_t* cap, void* out16, float* part, int32_t B,
                                int32_t Hq, int32_t Hkv, int32_t d, int32_t S, int32_t max_len, int32_t packed_out,
                                void* stream) {
  if (bad_dtype(dtype) || !qkv16 || !kv || !len_before || !kv_off || !cap || !out16 || B < 0 || Hq < 1 || Hkv < 1 ||
      Hq % Hkv || (d != 64 && d != 128) || S < 0 || S > 16)
    return SN_E_INVAL;
  if (S == 0) {
    if (max_len < 1) return SN_E_INVAL;
    S = attn_decode_splits(B, Hkv, max_len);
  }
  if (S > 1 && !part) return SN_E_INVAL;
  StepIndex ix{};
  ix.len_before = len_before;
  ix.kv_off = kv_off;
  ix.cap = cap;
  return rc_of(launch_attn_decode(dtype, qkv16, kv, ix, out16, part, B, Hq, Hkv, d, S, (hipStream_t)stream, packed_out != 0));
}

extern "C" int sn_k_attn_decode_append(int32_t dtype, const void* qkv16, void* kv, void* mirror, const float* inv_freq,
                                       int32_t rope, const int32_t* len_before, const int32_t* kv_off,
                                       const int32_t* cap, void* out16, float* part, int32_t B, int32_t Hq,
                                       int32_t Hkv, int32_t d, int32_t S, int32_t max_len, int32_t packed_out,
                                       void* stream) {
  if (bad_dtype(dtype) || !qkv16 || !kv || !len_before || !kv_off || !cap || !out16 || B < 0 || Hq < 1 || Hkv < 1 ||
      Hq % Hkv || (d != 64 && d != 128) || S < 0 || S > 16 || (rope && !inv_freq))
    return SN_E_INVAL;
  if (S == 0) {
    if (max_len < 1) return SN_E_INVAL;
    S = attn_decode_splits(B, Hkv, max_len);
  }
  if (S > 1 && !part) return SN_E_INVAL;
  StepIndex ix{};
  ix.len_before = len_before;
  ix.kv_off = kv_off;
  ix.cap = cap;
  const AttnAppend ap{(uint16_t*)kv, (uint16_t*)mirror, inv_freq, rope ? 1 : 0};
  return rc_of(launch_attn_decode(dtype, qkv16, kv, ix, out16, part, B, Hq, Hkv, d, S, (hipStream_t)stream,
                                  packed_out != 0, &ap));
}

extern "C" int sn_k_attn_decode_append_planes(int32_t dtype, const float* qkv_part, int32_t splits, int32_t plane_rows,
                                              void* kv, void* mirror, const float* inv_freq, int32_t rope,
                                              const int32_t* len_before, const int32_t* kv_off, const int32_t* cap,
                                              void* out16, float* part, int32_t B, int32_t Hq, int32_t Hkv, int32_t d,
                                              int32_t S, int32_t max_len, int32_t packed_out, void* stream) {
  if (bad_dtype(dtype) || !qkv_part || splits < 1 || splits > kMaxSplits || plane_rows < B || !kv || !len_before ||
      !kv_off || !cap || !out16 || B < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv || (d != 64 && d != 128) || S < 0 || S > 16 ||
      (rope && !inv_freq))
    return SN_E_INVAL;
  if (S == 0) {
    if (max_len < 1) return SN_E_INVAL;
    S = attn_decode_splits(B, Hkv, max_len);
  }
  if (S > 1 && !part) return SN_E_INVAL;
  StepIndex ix{};
  ix.len_before = len_before;
  ix.kv_off = kv_off;
  ix.cap = cap;
  AttnAppend ap{(uint16_t*)kv, (uint16_t*)mirror, inv_freq, rope ? 1 : 0};
  ap.qkv_part = qkv_part;
  ap.qkv_nsplit = splits;
  ap.qkv_rows = plane_rows;
  return rc_of(launch_attn_decode(dtype, nullptr, kv, ix, out16, part, B, Hq, Hkv, d, S, (hipStream_t)stream,
                                  packed_out != 0, &ap));
}

extern "C" int sn_k_attn_prefill(int32_t dtype, const void* qkv16, const void* kv, const int32_t* len_before,
                                 const int32_t* n_new, const int32_t* tok_start, const int32_t* kv_off,
                                 const int32_t* cap, const int32_t* tile_seq, const int32_t* tile_q0, void* out16,
                                 int32_t n_qtiles, int32_t Hq, int32_t Hkv, int32_t d, int32_t packed_out, void* stream) {
  if (bad_dtype(dtype) || !qkv16 || !kv || !len_before || !n_new || !tok_start || !kv_off || !cap || !tile_seq ||
      !tile_q0 || !out16 || n_qtiles < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv || (d != 64 && d != 128))
    return SN_E_INVAL;
  StepIndex ix{};
  ix.len_before = len_before;
  ix.n_new = n_new;
  ix.tok_start = tok_start;
  ix.kv_off = kv_off;
  ix.cap = cap;
  ix.tile_seq = tile_seq;
  ix.tile_q0 = tile_q0;
  return rc_of(launch_attn_prefill(dtype, qkv16, kv, ix, out16, n_qtiles, Hq, Hkv, d, (hipStream_t)stream, packed_out != 0));
}

extern "C" int sn_k_cast_in(int32_t dtype, const void* in16, void* x32, uint64_t n, void* stream) {
  if (bad_dtype(dtype) || !in16 || !x32) return SN_E_INVAL;
  return rc_of(launch_cast_in(dtype, in16, (float*)x32, n, (hipStream_t)stream));
}
extern "C" int sn_k_cast_out(int32_t dtype, const void* x32, void* out16, uint64_t n, void* stream) {
  if (bad_dtype(dtype) || !x32 || !out16) return SN_E_INVAL;
  return rc_of(launch_cast_out(dtype, (const float*)x32, out16, n, (hipStream_t)stream));
}

extern "C" int sn_k_copy(const void* src, void* dst, uint64_t bytes, void* stream) {
  if (!src || !dst || bytes % 16) return SN_E_INVAL;
  return rc_of(launch_copy(src, dst, bytes, (hipStream_t)stream));
}

extern "C" int sn_k_gemm_splitk(int32_t dtype, const void* W, const void* X, const void* bias, void* part, int32_t M,
                                int32_t N, int32_t K, int32_t splits, int32_t flags, void* stream) {
  if (bad_dtype(dtype) || !W || !X || !part || M < 0 || M > kMaxDecodeRows || N < 16 || K < 32 || (flags & ~1)) return SN_E_INVAL;
  if (splits == 0) splits = gemm_skinny_splits(M, N, K);
  if (splits < 1 || splits > kMaxSplits) return SN_E_INVAL;
  const hipError_t e = launch_gemm_skinny(dtype, EPI_PART32, W, X, bias, part, M, N, K, (hipStream_t)stream, splits, flags & 1 ? kXPacked : 0);
  return e == hipSuccess ? splits : rc_of(e);
}

extern "C" int sn_k_norm_fold(int32_t dtype, int32_t is_ln, void* x32, const void* gain, const void* shift, void* out16,
                              int32_t T, int32_t h, float eps, const void* part, int32_t splits, const void* bias,
                              int32_t packed_out, void* stream) {
  if (bad_dtype(dtype) || !x32 || !gain || !out16 || T < 0 || h < 1 || (is_ln && !shift) || splits < 0 ||
      splits > kMaxSplits || (splits > 0 && !part))
    return SN_E_INVAL;
  Fold f;
  f.part = (const float*)part;
  f.nsplit = splits;
  f.bias = bias;
  return rc_of(launch_norm_fold(dtype, is_ln, (float*)x32, gain, shift, out16, T, h, eps, f, (hipStream_t)stream, packed_out != 0));
}

extern "C" int sn_k_cast_out_fold(int32_t dtype, void* x32, void* out16, int32_t T, int32_t h, const void* part,
                                  int32_t splits, const void* bias, void* stream) {
  if (bad_dtype(dtype) || !x32 || !out16 || T < 0 || h < 4 || splits < 1 || splits > kMaxSplits || !part) return SN_E_INVAL;
  Fold f;
  f.part = (const float*)part;
  f.nsplit = splits;
  f.bias = bias;
  return rc_of(launch_cast_out_fold(dtype, dtype, (float*)x32, out16, T, h, f, (hipStream_t)stream));
}
