// Decode-phase projection: out = epilogue(X[M][K] * W^T) for M <= 64 token rows.
//
// The paper notes that decoding is memory-intensive (Sec. 2.1): each weight is used
// once per token row, so the kernel is a weight stream bounded by HBM bandwidth.
// Weights are stored as 16x32 tiles in matrix-core lane order, tile (nb, kb) at
// ((nb * K/32) + kb) * 1 KiB, so a wavefront reads each tile as one fully coalesced
// 1 KiB request and feeds it straight to v_mfma_f32_16x16x32 as the A operand
// (16 output features x 32 inputs); the B operand is the activation tile
// (32 inputs x 16 token rows).  One workgroup owns 16 output features (or a gate/up
// pair of 16 for SwiGLU); its KS wavefronts split K into contiguous ranges and their
// fp32 partial tiles are summed through LDS in a fixed order (deterministic).
#include "common.h"
#include "kernels.h"

namespace sn {

template <class T, int MT, int EPI>
__global__ __launch_bounds__(1024) void gemm_skinny_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ X, const uint16_t* __restrict__ bias,
    void* __restrict__ out, int M, int N, int K) {
  constexpr bool DUAL = EPI == EPI_SWIGLU16;
  constexpr int NW = DUAL ? 2 : 1;          // weight tiles per k-block
  extern __shared__ float red[];            // [KS][MT*NW][64][4]
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int KS = blockDim.x >> 6;
  const int KB = K >> 5;
  const int per = (KB + KS - 1) / KS;
  const int kb0 = wave * per;
  const int kb1 = min(KB, kb0 + per);
  const int nb = blockIdx.x;                // output block (16 columns of the result)

  const uint16_t* w0 = W + ((size_t)(nb * NW) * KB) * 512 + lane * 8;
  const uint16_t* w1 = w0 + (size_t)KB * 512;

  // activation rows this lane supplies (B operand: column = token row, 8 consecutive k)
  const uint16_t* xrow[MT];
  bool xok[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = mt * 16 + (lane & 15);
    xok[mt] = m < M;
    xrow[mt] = X + (size_t)(xok[mt] ? m : 0) * K + (lane >> 4) * 8;
  }

  f32x4 acc[MT][NW];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NW; ++j) acc[mt][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  constexpr int U = 4;
  int kb = kb0;
  for (; kb + U <= kb1; kb += U) {
    u16x8 a0[U], a1[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      a0[u] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(w0 + (size_t)(kb + u) * 512));
      if (DUAL) a1[u] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(w1 + (size_t)(kb + u) * 512));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        u16x8 b = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
        if (xok[mt]) b = *reinterpret_cast<const u16x8*>(xrow[mt] + (size_t)(kb + u) * 32);
        acc[mt][0] = mma16x16x32<T>(a0[u], b, acc[mt][0]);
        if (DUAL) acc[mt][NW - 1] = mma16x16x32<T>(a1[u], b, acc[mt][NW - 1]);
      }
    }
  }
  for (; kb < kb1; ++kb) {
    const u16x8 a0 = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(w0 + (size_t)kb * 512));
    u16x8 a1 = a0;
    if (DUAL) a1 = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(w1 + (size_t)kb * 512));
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      u16x8 b = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
      if (xok[mt]) b = *reinterpret_cast<const u16x8*>(xrow[mt] + (size_t)kb * 32);
      acc[mt][0] = mma16x16x32<T>(a0, b, acc[mt][0]);
      if (DUAL) acc[mt][NW - 1] = mma16x16x32<T>(a1, b, acc[mt][NW - 1]);
    }
  }

  // fixed-order reduction of the KS partial tiles
  constexpr int NACC = MT * NW;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NW; ++j)
      *reinterpret_cast<f32x4*>(red + ((size_t)(wave * NACC + mt * NW + j) * 64 + lane) * 4) = acc[mt][j];
  __syncthreads();

  for (int mt = wave; mt < MT; mt += KS) {
    f32x4 s[NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) {
      s[j] = f32x4{0.f, 0.f, 0.f, 0.f};
      for (int w = 0; w < KS; ++w)
        s[j] += *reinterpret_cast<const f32x4*>(red + ((size_t)(w * NACC + mt * NW + j) * 64 + lane) * 4);
    }
    const int m = mt * 16 + (lane & 15);
    if (m >= M) continue;
    const int nl = (lane >> 4) * 4;                  // first of this lane's 4 columns in the block
    const int n = nb * 16 + nl;                      // result column
    if (EPI == EPI_SWIGLU16) {
      const int F = N >> 1;
      u16x4 o;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float g = s[0][i], u = s[NW - 1][i];
        if (bias) {
          g += to_f32<T>(bias[n + i]);
          u += to_f32<T>(bias[F + n + i]);
        }
        o[i] = from_f32<T>(silu(g) * u);
      }
      *reinterpret_cast<u16x4*>(static_cast<uint16_t*>(out) + (size_t)m * F + n) = o;
    } else if (EPI == EPI_RESID32) {
      float* xr = static_cast<float*>(out) + (size_t)m * N + n;
      f32x4 r = *reinterpret_cast<const f32x4*>(xr);
#pragma unroll
      for (int i = 0; i < 4; ++i) r[i] += s[0][i] + (bias ? to_f32<T>(bias[n + i]) : 0.f);
      *reinterpret_cast<f32x4*>(xr) = r;
    } else {
      u16x4 o;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float v = s[0][i] + (bias ? to_f32<T>(bias[n + i]) : 0.f);
        if (EPI == EPI_GELU16) v = gelu_erf(v);
        o[i] = from_f32<T>(v);
      }
      *reinterpret_cast<u16x4*>(static_cast<uint16_t*>(out) + (size_t)m * N + n) = o;
    }
  }
}

// K-split per workgroup: enough wavefronts in flight to cover HBM latency on 256 CUs
// (target ~4096 wavefronts), a power of two in [4, 16], never more than K/32 blocks
// allow usefully, and at least as many as the epilogue needs.
static int pick_ks(int n_blocks, int KB) {
  int ks = 4;
  while (ks < 16 && n_blocks * ks < 4096) ks <<= 1;
  while (ks > 4 && ks > KB) ks >>= 1;
  return ks;
}

template <class T, int MT>
static hipError_t launch_mt(int epi, const uint16_t* W, const uint16_t* X, const uint16_t* bias, void* out,
                            int M, int N, int K, hipStream_t st) {
  const int KB = K / 32;
  const int nblk = epi == EPI_SWIGLU16 ? N / 32 : N / 16;
  const int ks0 = pick_ks(nblk, KB);
  const int nacc = MT * (epi == EPI_SWIGLU16 ? 2 : 1);
  int ks = ks0;
  while (ks * nacc > 64) ks >>= 1;          // partial tiles must fit 64 KiB of LDS
  const size_t lds = (size_t)ks * nacc * 64 * 4 * sizeof(float);
  dim3 grid(nblk), block(ks * 64);
  switch (epi) {
    case EPI_STORE16:
      hipLaunchKernelGGL((gemm_skinny_kernel<T, MT, EPI_STORE16>), grid, block, lds, st, W, X, bias, out, M, N, K);
      break;
    case EPI_GELU16:
      hipLaunchKernelGGL((gemm_skinny_kernel<T, MT, EPI_GELU16>), grid, block, lds, st, W, X, bias, out, M, N, K);
      break;
    case EPI_RESID32:
      hipLaunchKernelGGL((gemm_skinny_kernel<T, MT, EPI_RESID32>), grid, block, lds, st, W, X, bias, out, M, N, K);
      break;
    case EPI_SWIGLU16:
      hipLaunchKernelGGL((gemm_skinny_kernel<T, MT, EPI_SWIGLU16>), grid, block, lds, st, W, X, bias, out, M, N, K);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <class T>
static hipError_t launch_t(int epi, const uint16_t* W, const uint16_t* X, const uint16_t* bias, void* out, int M,
                           int N, int K, hipStream_t st) {
  if (M <= 16) return launch_mt<T, 1>(epi, W, X, bias, out, M, N, K, st);
  if (M <= 32) return launch_mt<T, 2>(epi, W, X, bias, out, M, N, K, st);
  if (M <= 48) return launch_mt<T, 3>(epi, W, X, bias, out, M, N, K, st);
  return launch_mt<T, 4>(epi, W, X, bias, out, M, N, K, st);
}

hipError_t launch_gemm_skinny(int dtype, int epi, const void* W, const void* X, const void* bias, void* out,
                              int M, int N, int K, hipStream_t st) {
  if (M <= 0) return hipSuccess;
  if (M > 64 || N % 16 || K % 32 || (epi == EPI_SWIGLU16 && N % 32)) return hipErrorInvalidValue;
  if (dtype == 0)
    return launch_t<F16>(epi, (const uint16_t*)W, (const uint16_t*)X, (const uint16_t*)bias, out, M, N, K, st);
  return launch_t<BF16>(epi, (const uint16_t*)W, (const uint16_t*)X, (const uint16_t*)bias, out, M, N, K, st);
}

}  // namespace sn
