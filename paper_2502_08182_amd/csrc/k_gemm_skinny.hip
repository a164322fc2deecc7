// Decode-phase projection: out = epilogue(X[M][K] * W^T) for M <= 64 token rows.
//
// The paper notes that decoding is memory-intensive (Sec. 2.1): each weight is used
// once per token row, so the kernel is a weight stream bounded by HBM bandwidth.
// Weights are stored as 16x32 tiles in matrix-core lane order, tile (nb, kb) at
// ((nb * K/32) + kb) * 1 KiB, so a wavefront reads each tile as one fully coalesced
// 1 KiB request and feeds it straight to v_mfma_f32_16x16x32 as the A operand
// (16 output features x 32 inputs); the B operand is the activation tile
// (32 inputs x 16 token rows).  A wavefront owns 16*C output features.  The KS
// wavefronts of a workgroup form NWN columns of KS/NWN: wavefronts side by side cover
// adjacent feature groups over the SAME K range, so the activation fragments they
// read are the same ones at about the same time and come from the L1 cache instead of
// L2 (at 64 token rows the activation reads cost a fifth of the weight stream's rate
// otherwise); wavefronts of one column split K into contiguous ranges and their fp32
// partial tiles are summed through LDS in a fixed order (deterministic).
#include <algorithm>

#include "kernels.h"
#include "common.h"

namespace sn {

// MT: 16-row tiles of token rows; C: adjacent 16-column blocks per wavefront (each
// activation fragment read from L2 is reused for C weight tiles, keeping activation
// traffic at or below weight traffic for every M <= 64).
// WMAX: most wavefronts a workgroup of this instance may have (bounds the register budget:
// 16 -> 128 registers, 8 or fewer -> 256, which the 4-row-tile variants need to stay out of
// scratch memory).
// SHARE: the instance supports more than one column of wavefronts (NWN_ > 1); without it the
// column count is the constant 1, which saves the registers the 4-row-tile split-K variants need
// to keep four wavefronts per SIMD.
template <class T, int MT, int C, int EPI, int WMAX, bool SHARE>
__global__ __launch_bounds__(WMAX * 64) void gemm_skinny_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ X, const uint16_t* __restrict__ bias,
    void* __restrict__ out, int M, int N, int K, int xpacked, int opacked, int NWN_) {
  const int NWN = SHARE ? NWN_ : 1;
  constexpr bool DUAL = EPI == EPI_SWIGLU16;
  static_assert(!DUAL || C % 2 == 0, "SwiGLU needs gate/up pairs");
  constexpr int U = C >= 4 ? 1 : (C == 2 ? 2 : 4);     // k-blocks in flight per column block
  constexpr bool SPLIT_ACC = MT * C == 1;              // lone accumulator: alternate two to hide MFMA latency
  extern __shared__ float red[];                       // [KS][C][64][4], reused for each row tile
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int KS = blockDim.x >> 6;
  const int KB = K >> 5;
  // K range of this workgroup (gridDim.y > 1 only for EPI_PART32), then of this wavefront
  const int per_wg = (KB + gridDim.y - 1) / gridDim.y;
  const int g0 = blockIdx.y * per_wg;
  const int g1 = min(KB, g0 + per_wg);
  const int wn = wave % NWN, wk = wave / NWN, KSK = KS / NWN;   // column of wavefronts, position in it
  const int per = (max(g1 - g0, 0) + KSK - 1) / KSK;
  const int kb0 = g0 + wk * per;
  const int kb1 = min(g1, kb0 + per);
  const int cb = (blockIdx.x * NWN + wn) * C;          // first 16-row block of the weight matrix

  const uint16_t* wp = W + ((size_t)cb * KB) * 512 + lane * 8;
  const size_t wstride = (size_t)KB * 512;             // next column block

  const uint16_t* xrow[MT];
  bool xok[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = mt * 16 + (lane & 15);
    xok[mt] = m < M;
    xrow[mt] = xpacked ? X + ((size_t)mt * KB * 64 + lane) * 8 : X + (size_t)(xok[mt] ? m : 0) * K + (lane >> 4) * 8;
  }
  const int xstep = xpacked ? 512 : 32;                // elements from one k-block to the next

  f32x4 acc[MT][C];
  f32x4 acc_b = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int c = 0; c < C; ++c) acc[mt][c] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Every wavefront walks its K range starting at a different rotation.  Tile rows of the
  // weight matrix lie a power of two apart, so wavefronts that all start at the beginning of
  // their range march over the HBM channels in lock-step (measured: 4.8 vs 6.1 TB/s on a
  // 4096 x 16384 matrix).  The rotation is a fixed function of (workgroup, K range), so the
  // summation order, and with it the result, stays reproducible -- and wavefronts side by side
  // walk the same k-blocks at the same time.
  const int len = max(kb1 - kb0, 0);
  const int rot = len > 0 ? ((blockIdx.x + wk * 5 + blockIdx.y * 3) * 4) % len : 0;
  for (int seg = 0; seg < 2; ++seg) {
    int kb = seg == 0 ? kb0 + rot : kb0;
    const int kend = seg == 0 ? kb1 : kb0 + rot;
    for (; kb + U <= kend; kb += U) {
      u16x8 a[U][C], b[U][MT];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < C; ++c)
          a[u][c] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(wp + c * wstride + (size_t)(kb + u) * 512));
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          b[u][mt] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
          if (xok[mt]) b[u][mt] = *reinterpret_cast<const u16x8*>(xrow[mt] + (size_t)(kb + u) * xstep);
        }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int c = 0; c < C; ++c) {
            if (SPLIT_ACC && (u & 1))
              acc_b = mma16x16x32<T>(a[u][c], b[u][mt], acc_b);
            else
              acc[mt][c] = mma16x16x32<T>(a[u][c], b[u][mt], acc[mt][c]);
          }
    }
    for (; kb < kend; ++kb) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        u16x8 b = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
        if (xok[mt]) b = *reinterpret_cast<const u16x8*>(xrow[mt] + (size_t)kb * xstep);
#pragma unroll
        for (int c = 0; c < C; ++c) {
          const u16x8 a = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(wp + c * wstride + (size_t)kb * 512));
          acc[mt][c] = mma16x16x32<T>(a, b, acc[mt][c]);
        }
      }
    }
  }
  if (SPLIT_ACC) acc[0][0] += acc_b;

  // fixed-order reduction of the KS partial tiles, one row tile at a time
  constexpr int ITEMS = DUAL ? C / 2 : C;              // epilogue work items per row tile
  const int nl = (lane >> 4) * 4;                      // first of this lane's 4 columns in a block
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if (mt) __syncthreads();
#pragma unroll
    for (int c = 0; c < C; ++c)
      *reinterpret_cast<f32x4*>(red + ((size_t)(wave * C + c) * 64 + lane) * 4) = acc[mt][c];
    __syncthreads();
    const int m = mt * 16 + (lane & 15);
    // epilogue work items: (column of wavefronts, output block [pair]); dealt round-robin to the wavefronts
    for (int item = wave; item < NWN * ITEMS; item += SHARE ? KS : ITEMS) {   // one pass at most when !SHARE
      if (m >= M) break;
      const int wn_i = item / ITEMS, it = item % ITEMS;
      const int cb_i = (blockIdx.x * NWN + wn_i) * C;
      const int c0 = DUAL ? it * 2 : it;
      f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = f32x4{0.f, 0.f, 0.f, 0.f};
      for (int w = 0; w < KSK; ++w) {
        s0 += *reinterpret_cast<const f32x4*>(red + ((size_t)((w * NWN + wn_i) * C + c0) * 64 + lane) * 4);
        if (DUAL) s1 += *reinterpret_cast<const f32x4*>(red + ((size_t)((w * NWN + wn_i) * C + c0 + 1) * 64 + lane) * 4);
      }
      if (EPI == EPI_SWIGLU16) {
        const int F = N >> 1;
        const int n = ((cb_i >> 1) + it) * 16 + nl;
        u16x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float g = s0[i], u = s1[i];
          if (bias) {
            g += to_f32<T>(bias[n + i]);
            u += to_f32<T>(bias[F + n + i]);
          }
          o[i] = from_f32<T>(silu(g) * u);
        }
        const size_t at = opacked ? packed_off(m, n, F >> 5) : (size_t)m * F + n;
        *reinterpret_cast<u16x4*>(static_cast<uint16_t*>(out) + at) = o;
      } else {
        const int n = (cb_i + c0) * 16 + nl;
        if (EPI == EPI_PART32) {
          // the bias goes into plane 0 here, not into the later fold: the fold runs inside the NEXT layer,
          // when this layer's weight record (a staging slot, if the layer is host-resident) may already
          // be receiving another layer
          if (bias && blockIdx.y == 0)
#pragma unroll
            for (int i = 0; i < 4; ++i) s0[i] += to_f32<T>(bias[n + i]);
          *reinterpret_cast<f32x4*>(static_cast<float*>(out) + ((size_t)blockIdx.y * M + m) * N + n) = s0;
        } else if (EPI == EPI_RESID32) {
          float* xr = static_cast<float*>(out) + (size_t)m * N + n;
          f32x4 r = *reinterpret_cast<const f32x4*>(xr);
#pragma unroll
          for (int i = 0; i < 4; ++i) r[i] += s0[i] + (bias ? to_f32<T>(bias[n + i]) : 0.f);
          *reinterpret_cast<f32x4*>(xr) = r;
        } else {
          u16x4 o;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float v = s0[i] + (bias ? to_f32<T>(bias[n + i]) : 0.f);
            if (EPI == EPI_GELU16) v = gelu_erf(v);
            o[i] = from_f32<T>(v);
          }
          const size_t at = opacked ? packed_off(m, n, N >> 5) : (size_t)m * N + n;
          *reinterpret_cast<u16x4*>(static_cast<uint16_t*>(out) + at) = o;
        }
      }
    }
  }
}

// K-split per workgroup (wavefronts per workgroup).  Measured on MI355X with M = 8:
// 8 wavefronts reach 6.0-6.2 TB/s on [12288|16384] x 4096 and 5.2 TB/s on 4096 x 4096;
// 16 are better (5.35 vs 5.0 TB/s) only when few column groups meet a long K
// (4096 x 16384).  Never fewer wavefronts than epilogue items (C <= 4).
static int pick_ks(int groups, int KB) {
  int ks = 8;
  if (groups * ks < 4096 && KB / (2 * ks) >= 16) ks = 16;
  return ks;
}

// Columns of wavefronts that share their activation reads (see the kernel).  Measured at 64 rows:
// 57344 x 8192 4.9 -> 5.9 TB/s, at 32 rows: 27648 x 5120 4.8 -> 5.7 TB/s.  More columns mean fewer
// workgroups, and what decides then is how evenly they fill the 256 compute units: 336 workgroups
// (one unit in three holds two) ran 21504 x 7168 at 32 rows in 77 us where 672 take 62.  So: the
// widest sharing among the counts that fill the chip about as evenly as any, never below 128
// workgroups.  At 16 rows or fewer the wavefronts of a column must also keep a long K run each
// (>= 128 k-blocks; 28672 x 7168: 6.0 -> 6.4 TB/s), or the shorter kernels lose more at start-up
// than the reads gain.
static int pick_columns(int MT, int groups, int KB, int ks) {
  auto evenness = [](int wgs) { return (double)wgs / (double)((wgs + 255) / 256 * 256); };
  double best = evenness(groups);
  for (int nwn = 2; nwn <= (MT == 1 ? 8 : 4); nwn <<= 1)
    if (ks % nwn == 0 && groups % nwn == 0 && groups / nwn >= 128) best = std::max(best, evenness(groups / nwn));
  for (int nwn = MT == 1 ? 8 : 4; nwn > 1; nwn >>= 1) {
    if (ks % nwn || groups % nwn || groups / nwn < 128) continue;
    if (MT == 1 && KB * nwn / ks < 128) continue;
    if (evenness(groups / nwn) >= best - 0.03) return nwn;
  }
  return 1;
}

template <class T, int MT, int C, int WMAX, bool SHARE>
static hipError_t launch_w(int epi, int ks, int nwn, const uint16_t* W, const uint16_t* X, const uint16_t* bias, void* out,
                           int M, int N, int K, int splits, int xpacked, int opacked, hipStream_t st) {
  const int groups = N / (16 * C * nwn);
  const size_t lds = (size_t)ks * C * 64 * 4 * sizeof(float);     // <= 64 KiB (ks <= 16, C <= 4)
  dim3 grid(groups, epi == EPI_PART32 ? splits : 1), block(ks * 64);
  if (ks > WMAX || ks % nwn || (N / (16 * C)) % nwn || (!SHARE && nwn != 1)) return hipErrorInvalidValue;
  switch (epi) {
    case EPI_PART32:
      SN_LAUNCH((gemm_skinny_kernel<T, MT, C, EPI_PART32, WMAX, SHARE>), grid, block, lds, st, W, X, bias, out, M, N, K, xpacked, opacked, nwn);
      break;
    case EPI_STORE16:
      SN_LAUNCH((gemm_skinny_kernel<T, MT, C, EPI_STORE16, WMAX, SHARE>), grid, block, lds, st, W, X, bias, out, M, N, K, xpacked, opacked, nwn);
      break;
    case EPI_GELU16:
      SN_LAUNCH((gemm_skinny_kernel<T, MT, C, EPI_GELU16, WMAX, SHARE>), grid, block, lds, st, W, X, bias, out, M, N, K, xpacked, opacked, nwn);
      break;
    case EPI_RESID32:
      SN_LAUNCH((gemm_skinny_kernel<T, MT, C, EPI_RESID32, WMAX, SHARE>), grid, block, lds, st, W, X, bias, out, M, N, K, xpacked, opacked, nwn);
      break;
    case EPI_SWIGLU16:
      if constexpr (C % 2 == 0) {
        SN_LAUNCH((gemm_skinny_kernel<T, MT, C, EPI_SWIGLU16, WMAX, SHARE>), grid, block, lds, st, W, X, bias, out, M, N, K, xpacked, opacked, nwn);
        break;
      }
      return hipErrorInvalidValue;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <class T, int MT, int C>
static hipError_t launch_mc(int epi, const uint16_t* W, const uint16_t* X, const uint16_t* bias, void* out,
                            int M, int N, int K, int splits, int xpacked, int opacked, hipStream_t st) {
  const int KB = K / 32;
  const int groups = N / (16 * C);
  if (epi == EPI_PART32) {
    // 3-4 row tiles, a long K per split and enough feature groups: 4 columns of 2 wavefronts
    // (64 rows, 8192 x 28672, 8 splits: 96 -> 87 us)
    if constexpr (MT >= 3 && C == 4)
      if (groups % 4 == 0 && groups / 4 * splits >= 200 && KB / splits >= 64)
        return launch_w<T, MT, C, 8, true>(epi, 8, 4, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
    // 3-4 row tiles otherwise: 8 wavefronts (few splits, see gemm_skinny_splits); up to 2 row tiles:
    // 4 wavefronts, the K split across workgroups provides the parallelism
    if constexpr (MT >= 3)
      return launch_w<T, MT, C, 8, false>(epi, 8, 1, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
    else
      return launch_w<T, MT, C, 16, false>(epi, (MT == 1 && splits == 1) ? 8 : 4, 1, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
  }
  if constexpr (MT >= 3) {      // 8 wavefronts at most: twice the registers, nothing spills
    const int nwn = pick_columns(MT, groups, KB, 8);
    if (nwn > 1) return launch_w<T, MT, C, 8, true>(epi, 8, nwn, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
    return launch_w<T, MT, C, 8, false>(epi, 8, 1, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
  } else {
    const int ks = pick_ks(groups, KB);
    const int nwn = pick_columns(MT, groups, KB, ks);
    if (nwn > 1) return launch_w<T, MT, C, 16, true>(epi, ks, nwn, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
    return launch_w<T, MT, C, 16, false>(epi, ks, 1, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
  }
}

// Column blocks per wavefront: as many as row tiles (activation traffic <= weight
// traffic), limited by what divides the number of 16-row weight blocks; SwiGLU needs
// an even count (gate/up pairs).
template <class T>
static hipError_t launch_t(int epi, const uint16_t* W, const uint16_t* X, const uint16_t* bias, void* out, int M,
                           int N, int K, int splits, int xpacked, int opacked, hipStream_t st) {
  const int nb = N / 16;
  const bool dual = epi == EPI_SWIGLU16;
  if (M <= 16) {
    if (dual) return launch_mc<T, 1, 2>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
    return launch_mc<T, 1, 1>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
  }
  if (M <= 32) {
    if (nb % 2 == 0) return launch_mc<T, 2, 2>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
    return launch_mc<T, 2, 1>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
  }
  if (M <= 48) {
    if (nb % 4 == 0) return launch_mc<T, 3, 4>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
    if (nb % 2 == 0) return launch_mc<T, 3, 2>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
    return launch_mc<T, 3, 1>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
  }
  if (nb % 4 == 0) return launch_mc<T, 4, 4>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
  if (nb % 2 == 0) return launch_mc<T, 4, 2>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
  return launch_mc<T, 4, 1>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, st);
}

hipError_t launch_gemm_skinny(int dtype, int epi, const void* W, const void* X, const void* bias, void* out,
                              int M, int N, int K, hipStream_t st, int splits, int flags) {
  const int xpacked = flags & kXPacked ? 1 : 0, opacked = flags & kOutPacked ? 1 : 0;
  if (opacked && (epi == EPI_RESID32 || epi == EPI_PART32)) return hipErrorInvalidValue;
  if (opacked && (epi == EPI_SWIGLU16 ? (N / 2) % 32 : N % 32)) return hipErrorInvalidValue;
  if (M <= 0) return hipSuccess;
  if (M > 64 || N % 16 || K % 32 || (epi == EPI_SWIGLU16 && N % 32)) return hipErrorInvalidValue;
  if (epi == EPI_PART32 ? (splits < 1 || splits > kMaxSplits) : splits != 1) return hipErrorInvalidValue;
  if (dtype == 0)
    return launch_t<F16>(epi, (const uint16_t*)W, (const uint16_t*)X, (const uint16_t*)bias, out, M, N, K, splits, xpacked, opacked, st);
  return launch_t<BF16>(epi, (const uint16_t*)W, (const uint16_t*)X, (const uint16_t*)bias, out, M, N, K, splits, xpacked, opacked, st);
}

// Split count for the residual projections of a decode step (few output features, long
// K).  Up to 32 rows: enough 256-thread workgroups that every CU holds several, each
// wavefront still streaming at least 4 KiB of weights.  Above 32 rows every split costs a
// plane of 64 x N partial sums, written here and read again by the fold, so: 8 splits where
// the 4-column instance applies (long K, see launch_mc), else as few as give about one
// workgroup per CU (64 rows, 8192 x 8192: 2 splits 30.7 us, 8 splits 33.5 us).
int gemm_skinny_splits(int M, int N, int K) {
  const int C = M <= 16 ? 1 : (M <= 32 ? 2 : 4);
  const int groups = N / (16 * C);
  const int KB = K / 32;
  int sp = 1;
  if (M > 32) {
    if (groups % 4 == 0 && groups / 4 * 8 >= 200 && KB / 8 >= 64) return 8;
    while (sp < kMaxSplits && groups * sp < 200 && KB / (sp * 2) >= 64) sp *= 2;
    return sp;
  }
  // one row tile and the feature groups alone fill the 256 CUs evenly (4096 features: one workgroup each): no
  // split across workgroups, 8 wavefronts split K inside the workgroup, and the fold reads one plane instead of
  // four (4096 x 16384 at 8 rows: 22.5 -> 21.7 us, decode step 3.105 -> 3.05 ms).  448 groups (7168 features)
  // would leave the CUs unevenly loaded and lose 13 %.
  if (M <= 16 && groups >= 256 && groups % 256 == 0) return 1;
  while (sp < kMaxSplits && groups * 4 * sp < 4096 && KB / (4 * sp * 2) >= 4) sp *= 2;
  return sp;
}

}  // namespace sn
