// Shared device-side helpers for the gfx950 kernels: 16-bit storage types, wave64
// reductions, vector typedefs for the matrix-core builtins.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace sn {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// ---- 16-bit storage <-> fp32 --------------------------------------------------
struct F16 {};
struct BF16 {};

template <class T> __device__ __forceinline__ float to_f32(uint16_t b);
template <> __device__ __forceinline__ float to_f32<F16>(uint16_t b) {
  return (float)__builtin_bit_cast(_Float16, b);
}
template <> __device__ __forceinline__ float to_f32<BF16>(uint16_t b) {
  return __builtin_bit_cast(float, (uint32_t)b << 16);
}

template <class T> __device__ __forceinline__ uint16_t from_f32(float v);
template <> __device__ __forceinline__ uint16_t from_f32<F16>(float v) {
  return __builtin_bit_cast(uint16_t, (_Float16)v);   // round to nearest even
}
template <> __device__ __forceinline__ uint16_t from_f32<BF16>(float v) {
  uint32_t u = __builtin_bit_cast(uint32_t, v);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                            // nearest even
  return (uint16_t)(u >> 16);
}

// ---- matrix-core step: D[16x16] += A[16x32] * B[32x16], fp32 accumulate ---------
// Lane l supplies A[row l%16][k = 8*(l/16) .. +8] and B[k = 8*(l/16) .. +8][col l%16];
// it receives D[rows 4*(l/16) .. +4][col l%16].
template <class T> __device__ __forceinline__ f32x4 mma16x16x32(u16x8 a, u16x8 b, f32x4 c);
template <> __device__ __forceinline__ f32x4 mma16x16x32<F16>(u16x8 a, u16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x4 mma16x16x32<BF16>(u16x8 a, u16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// ---- row-tile packed activations (decode path) ---------------------------------------
// Element (m, k) of an [M][K] activation matrix stored as 16-row x 32-k tiles in
// B-operand lane order: tile (m/16, k/32) at ((m/16)*(K/32) + k/32) KiB, inside it lane
// (m%16) + 16*((k%32)/8) holds 8 consecutive k.  A wavefront then reads one tile as 64
// consecutive 16-byte pieces instead of 16 row segments a power of two apart.
__device__ __forceinline__ size_t packed_off(int m, int k, int KB) {
  return ((((size_t)(m >> 4) * KB + (k >> 5)) * 64) + (m & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}

// Rotate the 8 halfwords of v left by 2*g elements (g in 0..3) with selects only, so that
// element e0 of the result is element (e0 + 2g) % 8 of v and can be indexed statically.
__device__ __forceinline__ u16x8 rot_pairs(u16x8 v, int g) {
  u32x4 w = __builtin_bit_cast(u32x4, v);
  if (g & 1) w = u32x4{w[1], w[2], w[3], w[0]};
  if (g & 2) w = u32x4{w[2], w[3], w[0], w[1]};
  return __builtin_bit_cast(u16x8, w);
}

// ---- wave64 reductions ----------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// GELU with the error function, 0.5 x (1 + erf(x / sqrt 2)).  erf by the five-term rational approximation of
// Abramowitz & Stegun (7.1.26): erf(z) = 1 - (a1 t + .. + a5 t^5) exp(-z^2), t = 1 / (1 + p z), z >= 0, absolute
// error <= 1.5e-7 -- a reciprocal, an exponential and seven multiply-adds instead of the library routine's two
// branches (a fifth of the 256 x 256 projection tile's time at K = 4096 went into its epilogue's erff).  Written
// with P E = 1 - erf(|z|) so that negative arguments do not cancel: gelu(x) = x - h for x >= 0, -h for x < 0,
// h = |x| P E / 2.  Against the float64 definition over [-12, 12]: 3.3e-7 absolute, the rounding of the result.
__device__ __forceinline__ float gelu_erf(float x) {
  const float ax = fabsf(x), z = ax * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, z, 1.0f));
  const float P = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float E = __builtin_amdgcn_exp2f(-z * z * 1.4426950408889634f);
  const float h = 0.5f * ax * P * E;
  return x >= 0.f ? x - h : -h;
}
__device__ __forceinline__ float silu(float x) { return x / (1.0f + __expf(-x)); }

}  // namespace sn

// Launch through this macro so that a pending LaunchEvents pair (kernels.h) is honoured.
#define SN_LAUNCH(kernel, grid, block, lds, stream, ...)                                            \
  do {                                                                                              \
    ::sn::LaunchEvents& le_ = ::sn::next_launch_events();                                           \
    if (le_.start) {                                                                                \
      hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, le_.start, le_.stop, 0, __VA_ARGS__); \
      le_ = ::sn::LaunchEvents{};                                                                   \
    } else {                                                                                        \
      hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                            \
    }                                                                                               \
  } while (0)
