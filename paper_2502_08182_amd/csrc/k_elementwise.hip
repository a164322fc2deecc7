// Small bandwidth-trivial kernels of the layer: casts between the 16-bit boundary
// type and the fp32 residual stream, the two normalisations, rotary embedding with
// the KV-cache append, and a hash fill used by the profiler for generated inputs.
#include <algorithm>
#include "kernels.h"
#include "common.h"

namespace sn {

#define SN_DISPATCH_T(dtype, ...)                   \
  do {                                              \
    if ((dtype) == 0) { using T = F16; __VA_ARGS__; } \
    else { using T = BF16; __VA_ARGS__; }           \
  } while (0)

// ---------------------------------------------------------------------------------
// flag (may be null): cleared here at the start of an iteration, set by the cast at its end when a hidden state is
// not finite -- a 16-bit hand-off that overflowed (|v| > 65504 in float16) reaches the fp32 residual stream as
// inf or NaN and stays there, so this one check at the end covers every hand-off of the iteration.
template <class T>
__global__ void cast_in_kernel(const uint16_t* __restrict__ in, float* __restrict__ x, size_t n, int32_t* __restrict__ flag) {
  if (flag && blockIdx.x == 0 && threadIdx.x == 0) *flag = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    x[i] = to_f32<T>(in[i]);
}
template <class T>
__global__ void cast_out_kernel(const float* __restrict__ x, uint16_t* __restrict__ out, size_t n, int32_t* __restrict__ flag) {
  bool bad = false;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const float v = x[i];
    bad |= !(fabsf(v) <= 3.0e38f);
    out[i] = from_f32<T>(v);
  }
  if (flag && bad) *flag = 1;
}
// Values in [-1, 1) from an integer hash of the element index (generated profiler inputs).
template <class T>
__global__ void fill_hash_kernel(uint16_t* __restrict__ out, size_t n, uint32_t seed) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    uint32_t v = (uint32_t)i * 2654435761u + seed;
    v ^= v >> 16; v *= 0x7feb352du; v ^= v >> 15; v *= 0x846ca68bu; v ^= v >> 16;
    out[i] = from_f32<T>((float)(v >> 8) * (1.0f / 8388608.0f) - 1.0f);
  }
}

// Plain device-to-device copy, 16 bytes per thread per trip: a kernel of exactly known
// HBM traffic (n bytes read, n written) against which hardware counters are calibrated.
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
  if (bytes == 0) return hipSuccess;
  if (bytes % 16) return hipErrorInvalidValue;
  const size_t n16 = bytes / 16;
  const unsigned grid = (unsigned)std::min<size_t>(2048, (n16 + 255) / 256);
  SN_LAUNCH(copy_kernel, dim3(grid), dim3(256), 0, st, (const u32x4*)src, (u32x4*)dst, n16);
  return hipGetLastError();
}

// Fill with a 32-bit pattern, 16 bytes per thread per trip (debug: poisoning a released staging slot).
__global__ __launch_bounds__(256) void fill_kernel(u32x4* __restrict__ dst, size_t n16, uint32_t pattern) {
  const u32x4 v = u32x4{pattern, pattern, pattern, pattern};
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = v;
}

hipError_t launch_fill(void* dst, size_t bytes, uint32_t pattern, hipStream_t st) {
  if (bytes == 0) return hipSuccess;
  if (bytes % 16) return hipErrorInvalidValue;
  const size_t n16 = bytes / 16;
  const unsigned grid = (unsigned)std::min<size_t>(2048, (n16 + 255) / 256);
  SN_LAUNCH(fill_kernel, dim3(grid), dim3(256), 0, st, (u32x4*)dst, n16, pattern);
  return hipGetLastError();
}

// Occupies a stream for about `ticks` periods of the constant-rate wall clock (debug: delaying one of the
// streams so that an ordering that usually holds by luck has to be enforced by its fence).  One wavefront;
// it leaves when the time is up or after max_trips sleeps, whichever comes first, so it always ends.
__global__ void delay_kernel(uint64_t ticks, int max_trips) {
  const uint64_t t0 = wall_clock64();
  for (int i = 0; i < max_trips; ++i) {
    if ((uint64_t)wall_clock64() - t0 >= ticks) break;
    __builtin_amdgcn_s_sleep(64);
  }
}

hipError_t launch_delay(uint64_t ticks, int max_trips, hipStream_t st) {
  if (ticks == 0 || max_trips < 1) return hipSuccess;
  SN_LAUNCH(delay_kernel, dim3(1), dim3(64), 0, st, ticks, max_trips);
  return hipGetLastError();
}

static inline int grid_for(size_t n, int block) {
  size_t g = (n + block - 1) / block;
  return (int)(g < 1 ? 1 : (g > 4096 ? 4096 : g));
}

hipError_t launch_cast_in(int dtype, const void* in16, float* x32, size_t n, hipStream_t st, int32_t* flag) {
  if (n == 0) return hipSuccess;
  SN_DISPATCH_T(dtype, SN_LAUNCH(cast_in_kernel<T>, dim3(grid_for(n, 256)), dim3(256), 0, st,
                                          (const uint16_t*)in16, x32, n, flag));
  return hipGetLastError();
}
hipError_t launch_cast_out(int dtype, const float* x32, void* out16, size_t n, hipStream_t st, int32_t* flag) {
  if (n == 0) return hipSuccess;
  SN_DISPATCH_T(dtype, SN_LAUNCH(cast_out_kernel<T>, dim3(grid_for(n, 256)), dim3(256), 0, st,
                                          x32, (uint16_t*)out16, n, flag));
  return hipGetLastError();
}
hipError_t launch_fill_hash(int dtype, void* out16, size_t n, uint32_t seed, hipStream_t st) {
  if (n == 0) return hipSuccess;
  SN_DISPATCH_T(dtype, SN_LAUNCH(fill_hash_kernel<T>, dim3(grid_for(n, 256)), dim3(256), 0, st,
                                          (uint16_t*)out16, n, seed));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Normalisation over the hidden dimension: one workgroup per token row, the row is read
// once into registers (float4 per thread per trip), fp32 statistics, 16-bit output.
// LayerNorm uses the two-pass (centred) variance.  BLOCK threads, at most MAXV float4
// per thread: 1024 x 4 covers hidden <= 16384 for the few rows of a decode step,
// 256 x 16 for the many rows of a prefill.
template <int BLOCK>
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();                 // red may still be read from a previous call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < BLOCK / 64; ++w) t += red[w];
  return t;
}

// x32 row element group idx (4 floats) after folding pending split-K partials:
// x += bias + part[0] + part[1] + ... (fixed order).
template <class T>
__device__ __forceinline__ f32x4 folded(f32x4 v, const float* __restrict__ part, int nsplit, size_t split_stride,
                                        size_t off, const uint16_t* __restrict__ bias, int col) {
  if (bias) {
    const u16x4 b = *reinterpret_cast<const u16x4*>(bias + col);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += to_f32<T>(b[e]);
  }
  // partials are requested four at a time before the first of them is added (one memory latency
  // per group, not per partial); the additions keep their fixed order
  static_assert(kMaxSplits % 4 == 0, "groups of four");
#pragma unroll
  for (int s0 = 0; s0 < kMaxSplits; s0 += 4) {
    if (s0 >= nsplit) break;
    f32x4 p[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
      if (s0 + s < nsplit) p[s] = *reinterpret_cast<const f32x4*>(part + (size_t)(s0 + s) * split_stride + off);
#pragma unroll
    for (int s = 0; s < 4; ++s)
      if (s0 + s < nsplit) v += p[s];
  }
  return v;
}

template <class T, bool LN, int BLOCK, int MAXV, bool FOLD>
__global__ __launch_bounds__(BLOCK) void norm_kernel(float* __restrict__ x,
                                                     const uint16_t* __restrict__ gain,
                                                     const uint16_t* __restrict__ shift,
                                                     uint16_t* __restrict__ u, int h, float eps,
                                                     const float* __restrict__ part, int nsplit,
                                                     const uint16_t* __restrict__ fbias, int packed, int tile_rows) {
  __shared__ float red[BLOCK / 64];
  // One workgroup per row.  tile_rows > 0 (many rows, packed output, no fold): the 16 rows of a row tile go to 16
  // workgroups of the same XCD -- consecutive workgroup ids are dealt round-robin to the 8 XCDs -- so that the
  // 16-byte pieces they contribute to each KiB of the packed layout meet in one L2 and leave as whole lines
  // (32768 x 5120: 361 -> 234 us; the row-major writer takes 163); tile_rows is the row count, the grid is padded to
  // whole groups of 8 tiles.
  int rowi = blockIdx.x;
  if (tile_rows > 0) {
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    rowi = ((xcd + 8 * (j >> 4)) << 4) + (j & 15);
    if (rowi >= tile_rows) return;
  }
  f32x4* row = reinterpret_cast<f32x4*>(x + (size_t)rowi * h);
  uint16_t* out = u + (size_t)rowi * h;
  const int nv = h >> 2;
  const float inv_h = 1.0f / (float)h;
  f32x4 v[MAXV];
  u16x4 gv[MAXV], bv[MAXV];
  float s = 0.f;
  // gains and shifts come from the layer's weight record (HBM, cold): fetch them together with
  // the row so that their latency does not follow the two reductions
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int idx = threadIdx.x + i * BLOCK;
    gv[i] = bv[i] = u16x4{0, 0, 0, 0};
    if (idx < nv) {
      gv[i] = *reinterpret_cast<const u16x4*>(gain + idx * 4);
      if (LN) bv[i] = *reinterpret_cast<const u16x4*>(shift + idx * 4);
    }
  }
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int idx = threadIdx.x + i * BLOCK;
    v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (idx < nv) {
      v[i] = row[idx];
      if (FOLD) {
        v[i] = folded<T>(v[i], part, nsplit, (size_t)gridDim.x * h, (size_t)rowi * h + idx * 4, fbias, idx * 4);
        row[idx] = v[i];
      }
    }
    s += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
  }
  float mu = 0.f;
  if (LN) mu = block_sum<BLOCK>(s, red) * inv_h;
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int idx = threadIdx.x + i * BLOCK;
    if (idx < nv) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float c = v[i][e] - mu;
        ss += c * c;
      }
    }
  }
  const float rstd = rsqrtf(block_sum<BLOCK>(ss, red) * inv_h + eps);
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int idx = threadIdx.x + i * BLOCK;
    if (idx < nv) {
      const u16x4 g = gv[i], b = bv[i];
      u16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float r = (v[i][e] - mu) * rstd * to_f32<T>(g[e]);
        if (LN) r += to_f32<T>(b[e]);
        o[e] = from_f32<T>(r);
      }
      if (packed)
        *reinterpret_cast<u16x4*>(u + packed_off(rowi, idx * 4, h >> 5)) = o;
      else
        *reinterpret_cast<u16x4*>(out + idx * 4) = o;
    }
  }
}

template <class T, bool LN, bool FOLD>
static void launch_norm_t(float* x32, const uint16_t* gain, const uint16_t* shift, uint16_t* u16, int Tn, int h,
                          float eps, const Fold& f, int packed, hipStream_t st) {
  const uint16_t* fb = (const uint16_t*)f.bias;
  if (Tn <= 128 && h <= 4096)
    SN_LAUNCH((norm_kernel<T, LN, 1024, 1, FOLD>), dim3(Tn), dim3(1024), 0, st, x32, gain, shift, u16, h, eps, f.part,
              f.nsplit, fb, packed, 0);
  else if (Tn <= 128 && h <= 8192)
    SN_LAUNCH((norm_kernel<T, LN, 1024, 2, FOLD>), dim3(Tn), dim3(1024), 0, st, x32, gain, shift, u16, h, eps, f.part,
              f.nsplit, fb, packed, 0);
  else if (Tn <= 128)
    SN_LAUNCH((norm_kernel<T, LN, 1024, 4, FOLD>), dim3(Tn), dim3(1024), 0, st, x32, gain, shift, u16, h, eps, f.part,
              f.nsplit, fb, packed, 0);
  else if (packed && !FOLD)      // prefill, packed output: row tiles kept within an XCD (see the kernel)
    SN_LAUNCH((norm_kernel<T, LN, 256, 16, FOLD>), dim3(((Tn + 127) / 128) * 128), dim3(256), 0, st, x32, gain, shift, u16, h,
              eps, f.part, f.nsplit, fb, packed, Tn);
  else
    SN_LAUNCH((norm_kernel<T, LN, 256, 16, FOLD>), dim3(Tn), dim3(256), 0, st, x32, gain, shift, u16, h, eps, f.part,
              f.nsplit, fb, packed, 0);
}

hipError_t launch_norm_fold(int dtype, int is_ln, float* x32, const void* gain, const void* shift, void* u16, int Tn,
                            int h, float eps, const Fold& fold, hipStream_t st, int packed) {
  if (Tn == 0) return hipSuccess;
  if (h % 4 || h > 16384 || (packed && h % 32)) return hipErrorInvalidValue;
  const bool f = fold.nsplit > 0;
  SN_DISPATCH_T(dtype, {
    const uint16_t* g = (const uint16_t*)gain;
    const uint16_t* b = is_ln ? (const uint16_t*)shift : nullptr;
    uint16_t* o = (uint16_t*)u16;
    if (is_ln && f) launch_norm_t<T, true, true>(x32, g, b, o, Tn, h, eps, fold, packed, st);
    else if (is_ln) launch_norm_t<T, true, false>(x32, g, b, o, Tn, h, eps, fold, packed, st);
    else if (f) launch_norm_t<T, false, true>(x32, g, b, o, Tn, h, eps, fold, packed, st);
    else launch_norm_t<T, false, false>(x32, g, b, o, Tn, h, eps, fold, packed, st);
  });
  return hipGetLastError();
}

hipError_t launch_norm(int dtype, int is_ln, const float* x32, const void* gain, const void* shift,
                       void* u16, int Tn, int h, float eps, hipStream_t st) {
  return launch_norm_fold(dtype, is_ln, const_cast<float*>(x32), gain, shift, u16, Tn, h, eps, Fold{}, st, 0);
}

// Fold pending partials into the residual stream, write it back and emit the 16-bit output.
template <class T, class TB>
__global__ __launch_bounds__(256) void cast_out_fold_kernel(float* __restrict__ x, uint16_t* __restrict__ out, int Tn,
                                                            int h, const float* __restrict__ part, int nsplit,
                                                            const uint16_t* __restrict__ fbias, int32_t* __restrict__ flag) {
  const size_t nv = (size_t)Tn * h / 4;
  bool bad = false;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (size_t)gridDim.x * 256) {
    f32x4 v = reinterpret_cast<f32x4*>(x)[i];
    v = folded<TB>(v, part, nsplit, (size_t)Tn * h, i * 4, fbias, (int)((i * 4) % h));
    reinterpret_cast<f32x4*>(x)[i] = v;
    u16x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      bad |= !(fabsf(v[e]) <= 3.0e38f);
      o[e] = from_f32<T>(v[e]);
    }
    reinterpret_cast<u16x4*>(out)[i] = o;
  }
  if (flag && bad) *flag = 1;
}

hipError_t launch_cast_out_fold(int dtype, int bias_dtype, float* x32, void* out16, int Tn, int h, const Fold& fold,
                                hipStream_t st, int32_t* flag) {
  if (Tn == 0) return hipSuccess;
  if (h % 4) return hipErrorInvalidValue;
  const size_t nv = (size_t)Tn * h / 4;
  const dim3 grid(grid_for(nv, 256)), block(256);
  const uint16_t* fb = (const uint16_t*)fold.bias;
#define SN_COF(TT, TB) \
  SN_LAUNCH((cast_out_fold_kernel<TT, TB>), grid, block, 0, st, x32, (uint16_t*)out16, Tn, h, fold.part, fold.nsplit, fb, flag)
  if (dtype == 0 && bias_dtype == 0) SN_COF(F16, F16);
  else if (dtype == 1 && bias_dtype == 0) SN_COF(BF16, F16);
  else if (dtype == 1 && bias_dtype == 1) SN_COF(BF16, BF16);
  else if (dtype == 0 && bias_dtype == 1) SN_COF(F16, BF16);
  else return hipErrorInvalidValue;
#undef SN_COF
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Rotary embedding (pairs i, i + d/2; angle = position * inv_freq[i]) on q and k, and
// append of the new k, v rows to the KV slice.  One thread per (token, head slot, 8 pairs).
// KVR is the value type of the cache: k and v are rounded to KVR and then stored in the
// container type T (a bfloat16-valued cache lives in float16 containers, which hold
// every bfloat16 value of moderate magnitude exactly).
template <class T, class KVR>
__global__ __launch_bounds__(256) void rope_append_kernel(
    uint16_t* __restrict__ qkv, const int32_t* __restrict__ tok_seq, const int32_t* __restrict__ tok_pos,
    const int32_t* __restrict__ kv_off, const int32_t* __restrict__ cap, uint16_t* __restrict__ kv,
    uint16_t* __restrict__ mirror, const float* __restrict__ inv_freq, int Tn, int Hq, int Hkv, int d,
    int rope) {
  // one thread per (token, head slot, 8 pairs): 16 bytes from each half of the head
  const int half = d >> 1;
  const int chunks = half >> 3;
  const int slots = Hq + 2 * Hkv;
  const size_t total = (size_t)Tn * slots * chunks;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int i0 = (int)(idx % chunks) * 8;
  const int hs = (int)((idx / chunks) % slots);
  const int t = (int)(idx / ((size_t)chunks * slots));
  uint16_t* row = qkv + ((size_t)t * slots + hs) * d;
  const u16x8 va = *reinterpret_cast<const u16x8*>(row + i0);
  const u16x8 vb = *reinterpret_cast<const u16x8*>(row + i0 + half);
  const int pos = tok_pos[t];
  const bool is_q = hs < Hq;
  if (is_q && !rope) return;                       // q stays as the projection wrote it
  u16x8 oa, ob;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float a = to_f32<T>(va[e]), b = to_f32<T>(vb[e]);
    if (rope && hs < Hq + Hkv) {
      float sn_, cs_;
      sincosf((float)pos * inv_freq[i0 + e], &sn_, &cs_);
      const float ra = a * cs_ - b * sn_;
      const float rb = a * sn_ + b * cs_;
      a = ra;
      b = rb;
    }
    if (!is_q) {
      a = to_f32<KVR>(from_f32<KVR>(a));
      b = to_f32<KVR>(from_f32<KVR>(b));
    }
    oa[e] = from_f32<T>(a);
    ob[e] = from_f32<T>(b);
  }
  if (is_q) {
    *reinterpret_cast<u16x8*>(row + i0) = oa;
    *reinterpret_cast<u16x8*>(row + i0 + half) = ob;
    return;
  }
  const int s = tok_seq[t];
  const int c = cap[s];
  const bool is_v = hs >= Hq + Hkv;
  const int g = is_v ? hs - Hq - Hkv : hs - Hq;
  const size_t off = (size_t)kv_off[s] * 2 * Hkv * d + ((size_t)(g * 2 + (is_v ? 1 : 0)) * c + pos) * d;
  *reinterpret_cast<u16x8*>(kv + off + i0) = oa;
  *reinterpret_cast<u16x8*>(kv + off + i0 + half) = ob;
  if (mirror) {
    *reinterpret_cast<u16x8*>(mirror + off + i0) = oa;
    *reinterpret_cast<u16x8*>(mirror + off + i0 + half) = ob;
  }
}

hipError_t launch_rope_append(int dtype, int kv_value_dtype, void* qkv16, const StepIndex& ix, void* kv,
                              void* mirror, const float* inv_freq, int Tn, int Hq, int Hkv, int d, int rope,
                              hipStream_t st) {
  if (d % 16) return hipErrorInvalidValue;          // 8 pairs (16 bytes of each half) per thread
  const size_t total = (size_t)Tn * (Hq + 2 * Hkv) * (d / 16);
  if (total == 0) return hipSuccess;
  const unsigned grid = (unsigned)((total + 255) / 256);
#define SN_ROPE(TT, RR)                                                                                     \
  SN_LAUNCH((rope_append_kernel<TT, RR>), dim3(grid), dim3(256), 0, st, (uint16_t*)qkv16, ix.tok_seq, \
                     ix.tok_pos, ix.kv_off, ix.cap, (uint16_t*)kv, (uint16_t*)mirror, inv_freq, Tn, Hq, Hkv, d, rope)
  if (dtype == 0 && kv_value_dtype == 0) SN_ROPE(F16, F16);
  else if (dtype == 0 && kv_value_dtype == 1) SN_ROPE(F16, BF16);
  else if (dtype == 1 && kv_value_dtype == 1) SN_ROPE(BF16, BF16);
  else return hipErrorInvalidValue;
#undef SN_ROPE
  return hipGetLastError();
}

}  // namespace sn
