// Prefill-phase projection: out = epilogue(X[M][K] * W^T) for many token rows.
//
// Prefill is the computation-intensive phase (paper Sec. 2.1): a dense contraction, so
// it runs on the matrix cores (v_mfma_f32_16x16x32, fp32 accumulate).  Weight tiles
// (16 features x 32 k) are stored in matrix-core lane order and are read straight from
// global memory into registers as the A operand (one coalesced 1 KiB request per tile);
// D[feature][token]: a lane ends up with 4 consecutive features of one token, which
// makes the row-major output store a short vector.
//
// Two kernels:
//  * gemm_tile_lds_kernel -- the fast path (N % 256 == 0, K % 64 == 0).  A 256-thread
//    workgroup computes 128 tokens x 256 features; each wavefront owns 128 x 64 of it
//    (32 accumulator tiles).  The activation slab (128 tokens x 64 k) is shared by the
//    four wavefronts, so it is staged through LDS, double-buffered, already permuted
//    into B-operand lane order (conflict-free 16-byte reads); weights are private to a
//    wavefront, so they bypass LDS and are double-buffered in registers.  Workgroups
//    are numbered so that the ones resident on one XCD at a time share weight columns
//    and token rows in that XCD's L2.
//  * gemm_tile_kernel -- any N % 16 == 0, K % 32 == 0: 128 x 128 per workgroup, both
//    operands read directly from global memory.
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


// ---------------------------------------------------------------------------------
// fast path
// ---------------------------------------------------------------------------------
template <class T, int EPI>
__global__ __launch_bounds__(256, 2) void gemm_tile_lds_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ X, const uint16_t* __restrict__ bias,
    void* __restrict__ out, int M, int N, int K, int NT, int TT) {
  constexpr int BM = 128, BK = 64;
  __shared__ __attribute__((aligned(16))) uint16_t xs[2][BM / 16][BK / 32][64][8];   // 2 x 16 KiB

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int KB = K >> 5;
  const int S = K / BK;

  // XCD-aware numbering: hardware deals consecutive workgroup ids round-robin to the 8
  // XCDs.  Each XCD gets a contiguous band of NT/8 feature tiles and walks the token
  // tiles for that band, so that the ~32-64 workgroups it runs at once share weights
  // (same band) and activations (same token tile) in its L2.
  int tn, tt;
  {
    const int id = blockIdx.x;
    if (NT % 8 == 0) {
      const int xcd = id & 7, j = id >> 3, band = NT >> 3;
      tn = xcd * band + j % band;
      tt = j / band;
    } else {
      tn = id % NT;
      tt = id / NT;
    }
  }
  const int t0 = tt * BM;
  const int nb0 = tn * 16 + wave * 4;                      // first of this wavefront's 4 feature blocks

  const uint16_t* wp = W + ((size_t)nb0 * KB) * 512 + lane * 8;
  const size_t wstride = (size_t)KB * 512;

  // activation staging: thread handles chunks (row = tid/8 + 32*i, 8 k at 8*(tid%8))
  const int xr0 = threadIdx.x >> 3, xkc = threadIdx.x & 7;
  const uint16_t* xg[4];
  bool xok[4];
  uint16_t* xl[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = xr0 + 32 * i;
    xok[i] = t0 + row < M;
    xg[i] = X + (size_t)(xok[i] ? t0 + row : 0) * K + xkc * 8;
    xl[i] = &xs[0][row >> 4][xkc >> 2][(row & 15) + 16 * (xkc & 3)][0];
  }
  constexpr int kStage = (BM / 16) * (BK / 32) * 64 * 8;    // elements per LDS stage

  f32x4 acc[4][8];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[j][i] = f32x4{0.f, 0.f, 0.f, 0.f};

  u16x8 a_cur[2][4], a_nxt[2][4], xv[4];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk)
#pragma unroll
    for (int j = 0; j < 4; ++j) a_cur[kk][j] = *reinterpret_cast<const u16x8*>(wp + j * wstride + (size_t)kk * 512);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    xv[i] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
    if (xok[i]) xv[i] = *reinterpret_cast<const u16x8*>(xg[i]);
    *reinterpret_cast<u16x8*>(xl[i]) = xv[i];
  }
  __syncthreads();

  for (int s = 0; s < S; ++s) {
    const int cur = s & 1;
    const bool more = s + 1 < S;
    if (more) {
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          a_nxt[kk][j] = *reinterpret_cast<const u16x8*>(wp + j * wstride + (size_t)((s + 1) * 2 + kk) * 512);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        xv[i] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
        if (xok[i]) xv[i] = *reinterpret_cast<const u16x8*>(xg[i] + (size_t)(s + 1) * BK);
      }
    }
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        u16x8 b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) b[i] = *reinterpret_cast<const u16x8*>(&xs[cur][h * 4 + i][kk][lane][0]);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[j][h * 4 + i] = mma16x16x32<T>(a_cur[kk][j], b[i], acc[j][h * 4 + i]);
      }
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < 4; ++i) *reinterpret_cast<u16x8*>(xl[i] + (cur ^ 1) * kStage) = xv[i];
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int j = 0; j < 4; ++j) a_cur[kk][j] = a_nxt[kk][j];
    }
    __syncthreads();
  }

  const int nl = (lane >> 4) * 4;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int t = t0 + i * 16 + (lane & 15);
    if (t >= M) continue;
    if (EPI == EPI_SWIGLU16) {
      const int F = N >> 1;
#pragma unroll
      for (int j = 0; j < 4; j += 2) {
        const int n = ((nb0 + j) >> 1) * 16 + nl;
        u16x4 o;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float g = acc[j][i][r], u = acc[j + 1][i][r];
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
      for (int j = 0; j < 4; ++j) {
        const int n = (nb0 + j) * 16 + nl;
        if (EPI == EPI_RESID32) {
          float* xr = static_cast<float*>(out) + (size_t)t * N + n;
          f32x4 r = *reinterpret_cast<const f32x4*>(xr);
#pragma unroll
          for (int q = 0; q < 4; ++q) r[q] += acc[j][i][q] + (bias ? to_f32<T>(bias[n + q]) : 0.f);
          *reinterpret_cast<f32x4*>(xr) = r;
        } else {
          u16x4 o;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float v = acc[j][i][q] + (bias ? to_f32<T>(bias[n + q]) : 0.f);
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
  if (N % 256 == 0 && K % 64 == 0) {
    const int NT = N / 256, TT = (M + 127) / 128;
    dim3 grid(NT * TT), block(256);
    switch (epi) {
      case EPI_STORE16:
        SN_LAUNCH((gemm_tile_lds_kernel<T, EPI_STORE16>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT);
        break;
      case EPI_GELU16:
        SN_LAUNCH((gemm_tile_lds_kernel<T, EPI_GELU16>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT);
        break;
      case EPI_RESID32:
        SN_LAUNCH((gemm_tile_lds_kernel<T, EPI_RESID32>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT);
        break;
      case EPI_SWIGLU16:
        SN_LAUNCH((gemm_tile_lds_kernel<T, EPI_SWIGLU16>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT);
        break;
      default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
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
