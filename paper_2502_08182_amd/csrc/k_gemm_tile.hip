// Prefill-phase projection: out = epilogue(X[M][K] * W^T) for many token rows.
//
// Prefill is the computation-intensive phase (paper Sec. 2.1): a dense contraction, so
// it runs on the matrix cores.  A 256-thread workgroup computes a 128 (tokens) x 128
// (features) tile; each of its 4 wavefronts owns 64 x 64 of it as 4 x 4 MFMA
// 16x16x32 accumulators.  Weight tiles (16 features x 32 k) are already stored in
// matrix-core lane order and are read straight into registers as the A operand;
// activation rows are read as the B operand (8 consecutive k per lane).
// D[feature][token]: a lane ends up with 4 consecutive features of one token, which
// makes the row-major output store a short vector.
#include "kernels.h"
#include "common.h"

namespace sn {

template <class T, int EPI>
__global__ __launch_bounds__(256) void gemm_tile_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ X, const uint16_t* __restrict__ bias,
    void* __restrict__ out, int M, int N, int K) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int KB = K >> 5;
  const int NB = N >> 4;
  const int nb0 = blockIdx.x * 8 + (wave & 1) * 4;       // first of 4 feature blocks
  const int t0 = blockIdx.y * 128 + (wave >> 1) * 64;    // first of 64 token rows

  const uint16_t* wp[4];
  bool wok[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    wok[i] = nb0 + i < NB;
    wp[i] = W + ((size_t)(wok[i] ? nb0 + i : 0) * KB) * 512 + lane * 8;
  }
  const uint16_t* xp[4];
  bool xok[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int t = t0 + j * 16 + (lane & 15);
    xok[j] = t < M;
    xp[j] = X + (size_t)(xok[j] ? t : 0) * K + (lane >> 4) * 8;
  }

  f32x4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int kb = 0; kb < KB; ++kb) {
    u16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const u16x8*>(wp[i] + (size_t)kb * 512);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      b[j] = *reinterpret_cast<const u16x8*>(xp[j] + (size_t)kb * 32);
      if (!xok[j]) b[j] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = mma16x16x32<T>(a[i], b[j], acc[i][j]);
  }

  const int nl = (lane >> 4) * 4;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int t = t0 + j * 16 + (lane & 15);
    if (t >= M) continue;
    if (EPI == EPI_SWIGLU16) {
      const int F = N >> 1;
#pragma unroll
      for (int i = 0; i < 4; i += 2) {
        if (!wok[i + 1]) continue;
        const int n = ((nb0 + i) >> 1) * 16 + nl;
        u16x4 o;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float g = acc[i][j][r], u = acc[i + 1][j][r];
          if (bias) {
            g += to_f32<T>(bias[n + r]);
            u += to_f32<T>(bias[F + n + r]);
          }
          o[r] = from_f32<T>(silu(g) * u);
        }
        *reinterpret_cast<u16x4*>(static_cast<uint16_t*>(out) + (size_t)t * F + n) = o;
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (!wok[i]) continue;
        const int n = (nb0 + i) * 16 + nl;
        if (EPI == EPI_RESID32) {
          float* xr = static_cast<float*>(out) + (size_t)t * N + n;
          f32x4 r = *reinterpret_cast<const f32x4*>(xr);
#pragma unroll
          for (int q = 0; q < 4; ++q) r[q] += acc[i][j][q] + (bias ? to_f32<T>(bias[n + q]) : 0.f);
          *reinterpret_cast<f32x4*>(xr) = r;
        } else {
          u16x4 o;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float v = acc[i][j][q] + (bias ? to_f32<T>(bias[n + q]) : 0.f);
            if (EPI == EPI_GELU16) v = gelu_erf(v);
            o[q] = from_f32<T>(v);
          }
          *reinterpret_cast<u16x4*>(static_cast<uint16_t*>(out) + (size_t)t * N + n) = o;
        }
      }
    }
  }
}

template <class T>
static hipError_t launch_t(int epi, const uint16_t* W, const uint16_t* X, const uint16_t* bias, void* out, int M,
                           int N, int K, hipStream_t st) {
  dim3 grid((N / 16 + 7) / 8, (M + 127) / 128), block(256);
  switch (epi) {
    case EPI_STORE16:
      SN_LAUNCH((gemm_tile_kernel<T, EPI_STORE16>), grid, block, 0, st, W, X, bias, out, M, N, K);
      break;
    case EPI_GELU16:
      SN_LAUNCH((gemm_tile_kernel<T, EPI_GELU16>), grid, block, 0, st, W, X, bias, out, M, N, K);
      break;
    case EPI_RESID32:
      SN_LAUNCH((gemm_tile_kernel<T, EPI_RESID32>), grid, block, 0, st, W, X, bias, out, M, N, K);
      break;
    case EPI_SWIGLU16:
      SN_LAUNCH((gemm_tile_kernel<T, EPI_SWIGLU16>), grid, block, 0, st, W, X, bias, out, M, N, K);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_gemm_tile(int dtype, int epi, const void* W, const void* X, const void* bias, void* out, int M,
                            int N, int K, hipStream_t st) {
  if (M <= 0) return hipSuccess;
  if (N % 16 || K % 32 || (epi == EPI_SWIGLU16 && N % 32)) return hipErrorInvalidValue;
  if (dtype == 0)
    return launch_t<F16>(epi, (const uint16_t*)W, (const uint16_t*)X, (const uint16_t*)bias, out, M, N, K, st);
  return launch_t<BF16>(epi, (const uint16_t*)W, (const uint16_t*)X, (const uint16_t*)bias, out, M, N, K, st);
}

}  // namespace sn
