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

// The fused epilogue of one (row tile, output block [pair]) item: s0 (and, SwiGLU, s1) hold the finished sums of
// this lane's 4 features nl .. nl + 3 of block c0 (c0 + 1) of column wn_i, for token row m.
template <class T, int C, int EPI>
__device__ __forceinline__ void epilogue_item(f32x4 s0, f32x4 s1, int m, int wn_i, int it, int nl, int NWN,
                                              const uint16_t* __restrict__ bias, void* __restrict__ out, int N,
                                              int opacked, int plane_rows) {
  constexpr bool DUAL = EPI == EPI_SWIGLU16;
  const int cb_i = (blockIdx.x * NWN + wn_i) * C;
  const int c0 = DUAL ? it * 2 : it;
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
      *reinterpret_cast<f32x4*>(static_cast<float*>(out) + ((size_t)blockIdx.y * plane_rows + m) * N + n) = s0;
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

// Fixed-order reduction of the KS partial tiles through LDS (one row tile at a time) and the fused epilogue.
// red: [KS][C][64][4] floats.  Wavefront (wk, wn) = (wave / NWN, wave % NWN) holds the partial sums of
// column blocks (blockIdx.x * NWN + wn) * C .. + C over the wk-th part of the workgroup's K range.
// With one wavefront per column (KS == NWN) there is nothing to reduce: every wavefront finishes its own
// blocks from registers (the same sums, 0 + x, so the bits do not depend on which way a launch went).
template <class T, int MT, int C, int EPI>
__device__ __forceinline__ void reduce_and_store(float* red, const f32x4 (&acc)[MT][C], int lane, int wave, int KS, int NWN,
                                                 const uint16_t* __restrict__ bias, void* __restrict__ out, int M, int N,
                                                 int opacked, int plane_rows) {
  constexpr bool DUAL = EPI == EPI_SWIGLU16;
  const int KSK = KS / NWN;
  constexpr int ITEMS = DUAL ? C / 2 : C;              // epilogue work items per row tile
  const int nl = (lane >> 4) * 4;                      // first of this lane's 4 columns in a block
  if (KS == NWN) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = mt * 16 + (lane & 15);
      if (m >= M) continue;
#pragma unroll
      for (int it = 0; it < ITEMS; ++it) {
        const int c0 = DUAL ? it * 2 : it;
        f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = f32x4{0.f, 0.f, 0.f, 0.f};
        s0 += acc[mt][c0];
        if (DUAL) s1 += acc[mt][DUAL ? c0 + 1 : c0];
        epilogue_item<T, C, EPI>(s0, s1, m, wave, it, nl, NWN, bias, out, N, opacked, plane_rows);
      }
    }
    return;
  }
  // fixed-order reduction of the KS partial tiles, one row tile at a time
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if (mt) __syncthreads();
#pragma unroll
    for (int c = 0; c < C; ++c)
      *reinterpret_cast<f32x4*>(red + ((size_t)(wave * C + c) * 64 + lane) * 4) = acc[mt][c];
    __syncthreads();
    const int m = mt * 16 + (lane & 15);
    // epilogue work items: (column of wavefronts, output block [pair]); dealt round-robin to the wavefronts
    for (int item = wave; item < NWN * ITEMS; item += KS) {
      if (m >= M) break;
      const int wn_i = item / ITEMS, it = item % ITEMS;
      const int c0 = DUAL ? it * 2 : it;
      f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = f32x4{0.f, 0.f, 0.f, 0.f};
      for (int w = 0; w < KSK; ++w) {
        s0 += *reinterpret_cast<const f32x4*>(red + ((size_t)((w * NWN + wn_i) * C + c0) * 64 + lane) * 4);
        if (DUAL) s1 += *reinterpret_cast<const f32x4*>(red + ((size_t)((w * NWN + wn_i) * C + c0 + 1) * 64 + lane) * 4);
      }
      epilogue_item<T, C, EPI>(s0, s1, m, wn_i, it, nl, NWN, bias, out, N, opacked, plane_rows);
    }
  }
}

// MT: 16-row tiles of token rows; C: adjacent 16-column blocks per wavefront (each
// activation fragment read from L2 is reused for C weight tiles, keeping activation
// traffic at or below weight traffic for every M <= 64).
// WMAX: most wavefronts a workgroup of this instance may have (bounds the register budget:
// 16 -> 128 registers, 8 or fewer -> 256, which the 4-row-tile variants need to stay out of
// scratch memory).
// SHARE: the instance supports more than one column of wavefronts (NWN_ > 1); without it the
// column count is the constant 1, which saves the registers the 4-row-tile split-K variants need
// to keep four wavefronts per SIMD.
// k-blocks a wavefront keeps in flight (depth of its register ring): the deepest of 8, 4, 3, 2 whose ring of
// C weight and MT activation fragments fits the register budget beside the MT*C accumulators, up to 8 KiB of
// weights per wavefront where a compute unit holds 16 wavefronts and 12 KiB where it holds 8.
constexpr int ring_depth(int MT, int C, int WMAX) {
  const int budget = (WMAX > 8 ? 128 : 256) - 40 - MT * C * 4;
  const int most = (WMAX > 8 ? 8 : 12) / C;
  for (int pd : {8, 4, 3, 2})
    if (pd <= most && pd * (C + MT) * 4 <= budget) return pd;
  return 2;
}

template <class T, int MT, int C, int EPI, int WMAX, bool SHARE>
__global__ __launch_bounds__(WMAX * 64) void gemm_skinny_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ X, const uint16_t* __restrict__ bias,
    void* __restrict__ out, int M, int N, int K, int xpacked, int opacked, int NWN_, int plane_rows) {
  const int NWN = SHARE ? NWN_ : 1;
  constexpr bool DUAL = EPI == EPI_SWIGLU16;
  static_assert(!DUAL || C % 2 == 0, "SwiGLU needs gate/up pairs");
  constexpr int PD = ring_depth(MT, C, WMAX);
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
  //
  // From two row tiles on the walk is software-pipelined over a ring of PD k-blocks: the loads of
  // k-block i + PD are issued right after the products of k-block i, so a wavefront always has
  // PD - 1 .. PD k-blocks (C KiB of weights each) on their way while it computes.
  const int len = max(kb1 - kb0, 0);
  const int rot = len > 0 ? ((blockIdx.x + wk * 5 + blockIdx.y * 3) * 4) % len : 0;
  if constexpr (MT == 1) {
    // One row tile: the wavefront requests U k-blocks (U KiB of consecutive weights per column block) in one
    // burst, then multiplies them; 16 wavefronts per compute unit overlap each other's bursts.  (Keeping the
    // requests of single k-blocks in flight across the products, as below, measured 10-25 % slower here.)
    constexpr int U = C == 2 ? 2 : 4;
    for (int seg = 0; seg < 2; ++seg) {
      int kb = seg == 0 ? kb0 + rot : kb0;
      const int kend = seg == 0 ? kb1 : kb0 + rot;
      for (; kb + U <= kend; kb += U) {
        u16x8 a[U][C], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int c = 0; c < C; ++c)
            a[u][c] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(wp + c * wstride + (size_t)(kb + u) * 512));
#pragma unroll
        for (int u = 0; u < U; ++u) {
          b[u] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
          if (xok[0]) b[u] = *reinterpret_cast<const u16x8*>(xrow[0] + (size_t)(kb + u) * xstep);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int c = 0; c < C; ++c) {
            if (SPLIT_ACC && (u & 1))
              acc_b = mma16x16x32<T>(a[u][c], b[u], acc_b);
            else
              acc[0][c] = mma16x16x32<T>(a[u][c], b[u], acc[0][c]);
          }
      }
      for (; kb < kend; ++kb) {
        u16x8 b = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
        if (xok[0]) b = *reinterpret_cast<const u16x8*>(xrow[0] + (size_t)kb * xstep);
#pragma unroll
        for (int c = 0; c < C; ++c) {
          const u16x8 a = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(wp + c * wstride + (size_t)kb * 512));
          acc[0][c] = mma16x16x32<T>(a, b, acc[0][c]);
        }
      }
    }
  } else {
    u16x8 a[PD][C], b[PD][MT];
    // Token rows beyond M are loaded like the others (from row 0 of a row-major X; from the padding rows a
    // packed X always has): a token row only ever reaches its own output row, and those are not stored.  So the
    // loop body has no branches, and the loads of later k-blocks stay in flight across the products.
    auto load = [&](int slot, int i) {       // k-block number i of the rotated walk into ring slot `slot`
      int kb = kb0 + rot + i;
      if (kb >= kb1) kb -= len;
  #pragma unroll
      for (int c = 0; c < C; ++c)
        a[slot][c] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(wp + c * wstride + (size_t)kb * 512));
  #pragma unroll
      for (int mt = 0; mt < MT; ++mt) b[slot][mt] = *reinterpret_cast<const u16x8*>(xrow[mt] + (size_t)kb * xstep);
    };
    auto products = [&](int slot) {
  #pragma unroll
      for (int mt = 0; mt < MT; ++mt)
  #pragma unroll
        for (int c = 0; c < C; ++c) {
          if (SPLIT_ACC && (slot & 1))
            acc_b = mma16x16x32<T>(a[slot][c], b[slot][mt], acc_b);
          else
            acc[mt][c] = mma16x16x32<T>(a[slot][c], b[slot][mt], acc[mt][c]);
        }
    };
    if (len >= PD) {
  #pragma unroll
      for (int sl = 0; sl < PD; ++sl) load(sl, sl);
      int i = 0;
      for (; i + 2 * PD <= len; i += PD) {   // the ring is full and stays full: no conditions in here
  #pragma unroll
        for (int sl = 0; sl < PD; ++sl) {
          products(sl);
          load(sl, i + PD + sl);
          __builtin_amdgcn_sched_barrier(0);   // keep this order: the compiler would otherwise gather all products
                                               // first and all loads last, which empties the ring every round
        }
      }
      // the ring holds k-blocks i .. i + PD - 1; fewer than PD are left to request
  #pragma unroll
      for (int sl = 0; sl < PD; ++sl) {
        products(sl);
        if (i + PD + sl < len) load(sl, i + PD + sl);
      }
      i += PD;
  #pragma unroll
      for (int sl = 0; sl < PD; ++sl)
        if (i + sl < len) products(sl);
    } else {
      for (int i = 0; i < len; ++i) {        // a K range shorter than the ring
        load(0, i);
        products(0);
      }
    }
  }
  if (SPLIT_ACC) acc[0][0] += acc_b;

  reduce_and_store<T, MT, C, EPI>(red, acc, lane, wave, KS, NWN, bias, out, M, N, opacked, plane_rows);
}

// ---------------------------------------------------------------------------------------------
// 3-4 row tiles (33..64 token rows), activations shared through LDS.
//
// With that many rows a wavefront of the kernel above issues as many activation loads as weight
// loads, and although they hit the L1 cache they cost: doubling them (two column blocks per
// wavefront instead of four) took the 57344 x 8192 projection from 164 to 191 us, i.e. the
// weight stream alone would take ~137 us (6.85 TB/s) and every "weights' worth" of activation
// loads adds 27 us.  Here the wavefronts of a workgroup that walk the same K range (NWN side by
// side, each with its own C column blocks) fetch each activation tile ONCE, together, into LDS
// -- 16-byte pieces dealt round-robin over their lanes, two k-blocks per step, double-buffered,
// one barrier per step -- and every wavefront reads its B operands from there.  Weights go
// global -> registers as before, two steps ahead.  X must be row-tile packed.
template <class T, int MT, int C, int EPI>
__global__ __launch_bounds__(512) void gemm_wide_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ X, const uint16_t* __restrict__ bias,
    void* __restrict__ out, int M, int N, int K, int opacked, int NWN, int plane_rows) {
  constexpr int KC = 2;                                // k-blocks per step (4 and 8 measured no better at one row tile)
  constexpr int TILES = KC * MT;                       // activation tiles (1 KiB) per step and K range
  constexpr int R = (TILES + 3) / 4;                   // 16-byte pieces per lane and step (NWN >= 4)
  extern __shared__ __attribute__((aligned(16))) float red[];   // stages during the walk, partial tiles afterwards
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int KS = blockDim.x >> 6;
  const int KB = K >> 5;
  const int per_wg = (KB + gridDim.y - 1) / gridDim.y;
  const int g0 = blockIdx.y * per_wg;
  const int g1 = min(KB, g0 + per_wg);
  const int wn = wave % NWN, wk = wave / NWN, KSK = KS / NWN;
  const int per = (max(g1 - g0, 0) + KSK - 1) / KSK;   // longest K range of the workgroup: its step count is everyone's
  const int kb0 = g0 + wk * per;
  const int kb1 = min(g1, kb0 + per);
  const int len = max(kb1 - kb0, 0);
  const int nsteps = (per + KC - 1) / KC;
  const int rot = len > 0 ? ((blockIdx.x + wk * 5 + blockIdx.y * 3) * 4) % len : 0;
  // k-block at position i of this wavefront's rotated walk; positions past the end give some valid block
  // (their loads are harmless, their products are skipped)
  auto kb_at = [&](int i) {
    int kb = kb0 + rot + min(i, max(len - 1, 0));
    if (kb >= kb1) kb -= len;
    return min(max(kb, 0), KB - 1);
  };
  const int cb = (blockIdx.x * NWN + wn) * C;
  const uint16_t* wp = W + ((size_t)cb * KB) * 512 + lane * 8;
  const size_t wstride = (size_t)KB * 512;
  const int mtiles = (M + 15) >> 4;
  uint16_t* stage = reinterpret_cast<uint16_t*>(red) + (size_t)wk * (2 * TILES * 512);   // this K range's two stages

  // this lane's pieces of a step: piece p = tile (p / 64) = (kc, mt), 16 bytes number p % 64 of it
  int ptile[R], poff[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int p = min((wn + r * NWN) * 64 + lane, TILES * 64 - 1);   // surplus lanes repeat the last piece
    ptile[r] = p >> 6;
    poff[r] = (p & 63) * 8;
  }

  f32x4 acc[MT][C];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int c = 0; c < C; ++c) acc[mt][c] = f32x4{0.f, 0.f, 0.f, 0.f};
  u16x8 a[2][KC][C], sreg[R];

  auto wload = [&](int slot, int step) {
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const size_t kb = (size_t)kb_at(step * KC + kc);
#pragma unroll
      for (int c = 0; c < C; ++c)
        a[slot][kc][c] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(wp + c * wstride + kb * 512));
    }
  };
  auto sload = [&](int step) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      // row tiles past the last one X holds (MT may exceed ceil(M / 16)) read the last real tile: never stored
      const int kc = ptile[r] / MT, mt = min(ptile[r] % MT, mtiles - 1);
      sreg[r] = *reinterpret_cast<const u16x8*>(X + ((size_t)mt * KB + kb_at(step * KC + kc)) * 512 + poff[r]);
    }
  };
  auto sstore = [&](int s) {
#pragma unroll
    for (int r = 0; r < R; ++r) *reinterpret_cast<u16x8*>(stage + (size_t)(s * TILES + ptile[r]) * 512 + poff[r]) = sreg[r];
  };
  auto products = [&](int slot, int s, int step) {
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      if (step * KC + kc < len) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const u16x8 bf = *reinterpret_cast<const u16x8*>(stage + (size_t)(s * TILES + kc * MT + mt) * 512 + lane * 8);
#pragma unroll
          for (int c = 0; c < C; ++c) acc[mt][c] = mma16x16x32<T>(a[slot][kc][c], bf, acc[mt][c]);
        }
      }
    }
  };
  // LDS writes of this wavefront done, then everyone's: a bare barrier (a fence would also wait for the loads in flight)
  auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

  sload(0);
  wload(0, 0);
  sstore(0);
  sload(1);
  wload(1, 1);
  lds_barrier();
  for (int j = 0; j < nsteps; j += 2) {
    products(0, 0, j);
    __builtin_amdgcn_sched_barrier(0);
    sstore(1);                 // activations of step j + 1, requested one half-trip ago
    sload(j + 2);
    wload(0, j + 2);
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();
    products(1, 1, j + 1);
    __builtin_amdgcn_sched_barrier(0);
    sstore(0);
    sload(j + 3);
    wload(1, j + 3);
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();
  }
  // the last barrier also says: nobody reads the stages any more
  reduce_and_store<T, MT, C, EPI>(red, acc, lane, wave, KS, NWN, bias, out, M, N, opacked, plane_rows);
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

// Shape of the launch for 3-4 row tiles (8 wavefronts per compute unit at most): C column blocks per
// wavefront, nwn wavefronts side by side, ksk wavefronts splitting K below each.  A compute unit streams
// weights at a rate that hardly depends on how the work is cut, so what counts is how many 16-column blocks
// the busiest unit gets: workgroups are dealt out over the 256 units, each bringing nwn * C blocks.
// 57344 rows in blocks of 64 make 896 groups -- 224 workgroups of 4 columns leave 32 units idle -- but as
// 1792 groups of 32 in workgroups of 7 columns they are exactly one workgroup per unit.  Ties: more column
// blocks per wavefront (fewer operand reads per weight), then wider workgroups.  nwn >= 4 selects the kernel
// that shares activations through LDS; nwn == 1 means "no such shape" (too few feature groups).
struct WidePlan {
  int C, nwn, ks;
};
static WidePlan plan_wide(int nb, int KB, int only_c = 0) {
  WidePlan best{nb % 4 == 0 ? 4 : (nb % 2 == 0 ? 2 : 1), 1, 8};
  long best_cost = -1;
  for (int C : {4, 2}) {
    if (nb % C || (only_c && C != only_c)) continue;
    const int groups = nb / C;
    for (int nwn = 4; nwn <= 8; ++nwn) {
      if (groups % nwn) continue;
      const int wgs = groups / nwn;
      if (wgs < 128) continue;
      int ksk = 8 / nwn;
      while (ksk > 1 && KB / ksk < 16) --ksk;
      const long cost = (long)((wgs + 255) / 256) * nwn * C;
      if (best_cost < 0 || cost < best_cost || (cost == best_cost && (C > best.C || (C == best.C && nwn > best.nwn)))) {
        best = WidePlan{C, nwn, nwn * ksk};
        best_cost = cost;
      }
    }
  }
  return best;
}

// Launch shape of a split-K projection (fp32 partial planes) at 9..128 rows, from timings of every legal
// shape on MI355X (the residual and QKV shapes of the 13B-, 30B- and 70B-shaped layers at 32 and 64 rows): one
// wavefront per column (no K split inside the workgroup), the splits across workgroups provide the
// parallelism, at most 256 workgroups -- one per compute unit; a second round costs more than anything else --
// and at least 8 feature blocks per workgroup (activations fetched once per 8 weight tiles).
//  * K up to 16384 (start-up and drain are a large share of a 12-50 us launch): as many workgroups as
//    possible, then as few planes as possible (64 rows, 10240 x 8192: 5 columns x 2 blocks, 4 splits, 256
//    workgroups 30 us where 160 workgroups of the unsplit kernel took 46; 8192 x 8192: 26 us against 28;
//    32 rows, 5120 x 13824: 25 us against 28.5).
//  * longer K: the stream is chip-bound from ~190 workgroups on; 16 feature blocks per workgroup and the
//    fewest planes that reach 190 (64 rows, 8192 x 28672: 6 splits, 192 workgroups 81 us; 8 splits, 256
//    workgroups 86 us; 32 rows, 7168 x 28672: 66 us against 82).
// splits == 0: no such shape (odd block counts, too few features); the caller falls back to the other kernel.
struct SplitPlan {
  int C, nwn, splits;
};
static SplitPlan plan_split(int M, int nb, int KB) {
  SplitPlan best{0, 0, 0};
  if (M <= 8 || M > kMaxDecodeRows) return best;
  const bool long_k = KB > 512;
  long best_key = -1;
  for (int C : {4, 2}) {      // equal keys: four blocks per wavefront
    if (nb % C || (M > 64 && C != 2)) continue;     // 6 and 8 row tiles exist with two blocks per wavefront only
    const int groups = nb / C;
    for (int nwn = 4; nwn <= 8; ++nwn) {
      if (groups % nwn || nwn * C < 8 || nwn * C > 20) continue;
      for (int sp = 1; sp <= kMaxSplits; ++sp) {
        const int wgs = groups / nwn * sp;
        if (wgs > 256 || (sp > 1 && KB / sp < 32)) continue;
        long key;
        if (long_k)      // reach 190 workgroups; then 16 blocks per workgroup, few planes, more workgroups
          key = wgs >= 190 ? 1000000L + (nwn * C == 16 ? 100000L : 0) + (kMaxSplits - sp) * 1000L + wgs : wgs;
        else             // most workgroups, then fewest planes, then more blocks per workgroup
          key = wgs * 10000L + (kMaxSplits - sp) * 100L + nwn * C;
        if (key > best_key) {
          best_key = key;
          best = SplitPlan{C, nwn, sp};
        }
      }
    }
  }
  if (best.splits && nb / (best.C * best.nwn) * best.splits < 120) return SplitPlan{0, 0, 0};
  return best;
}

template <class T, int MT, int C>
static hipError_t launch_wide(int epi, int ks, int nwn, const uint16_t* W, const uint16_t* X, const uint16_t* bias, void* out,
                              int M, int N, int K, int splits, int opacked, int plane_rows, hipStream_t st) {
  const int groups = N / (16 * C * nwn);
  const int ksk = ks / nwn;
  const size_t lds = std::max((size_t)ks * C * 64 * 4 * sizeof(float), (size_t)ksk * 2 * 2 * MT * 1024);
  dim3 grid(groups, epi == EPI_PART32 ? splits : 1), block(ks * 64);
  if (nwn < 4 || ks > 8 || ks % nwn || (N / (16 * C)) % nwn) return hipErrorInvalidValue;
  switch (epi) {
    case EPI_PART32:
      SN_LAUNCH((gemm_wide_kernel<T, MT, C, EPI_PART32>), grid, block, lds, st, W, X, bias, out, M, N, K, opacked, nwn, plane_rows);
      break;
    case EPI_STORE16:
      SN_LAUNCH((gemm_wide_kernel<T, MT, C, EPI_STORE16>), grid, block, lds, st, W, X, bias, out, M, N, K, opacked, nwn, plane_rows);
      break;
    case EPI_GELU16:
      SN_LAUNCH((gemm_wide_kernel<T, MT, C, EPI_GELU16>), grid, block, lds, st, W, X, bias, out, M, N, K, opacked, nwn, plane_rows);
      break;
    case EPI_SWIGLU16:
      SN_LAUNCH((gemm_wide_kernel<T, MT, C, EPI_SWIGLU16>), grid, block, lds, st, W, X, bias, out, M, N, K, opacked, nwn, plane_rows);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <class T, int MT, int C, int WMAX, bool SHARE>
static hipError_t launch_w(int epi, int ks, int nwn, const uint16_t* W, const uint16_t* X, const uint16_t* bias, void* out,
                           int M, int N, int K, int splits, int xpacked, int opacked, int plane_rows, hipStream_t st) {
  const int groups = N / (16 * C * nwn);
  const size_t lds = (size_t)ks * C * 64 * 4 * sizeof(float);     // <= 64 KiB (ks <= 16, C <= 4)
  dim3 grid(groups, epi == EPI_PART32 ? splits : 1), block(ks * 64);
  if (ks > WMAX || ks % nwn || (N / (16 * C)) % nwn || (!SHARE && nwn != 1)) return hipErrorInvalidValue;
  switch (epi) {
    case EPI_PART32:
      SN_LAUNCH((gemm_skinny_kernel<T, MT, C, EPI_PART32, WMAX, SHARE>), grid, block, lds, st, W, X, bias, out, M, N, K, xpacked, opacked, nwn, plane_rows);
      break;
    case EPI_STORE16:
      SN_LAUNCH((gemm_skinny_kernel<T, MT, C, EPI_STORE16, WMAX, SHARE>), grid, block, lds, st, W, X, bias, out, M, N, K, xpacked, opacked, nwn, plane_rows);
      break;
    case EPI_GELU16:
      SN_LAUNCH((gemm_skinny_kernel<T, MT, C, EPI_GELU16, WMAX, SHARE>), grid, block, lds, st, W, X, bias, out, M, N, K, xpacked, opacked, nwn, plane_rows);
      break;
    case EPI_RESID32:
      SN_LAUNCH((gemm_skinny_kernel<T, MT, C, EPI_RESID32, WMAX, SHARE>), grid, block, lds, st, W, X, bias, out, M, N, K, xpacked, opacked, nwn, plane_rows);
      break;
    case EPI_SWIGLU16:
      if constexpr (C % 2 == 0) {
        SN_LAUNCH((gemm_skinny_kernel<T, MT, C, EPI_SWIGLU16, WMAX, SHARE>), grid, block, lds, st, W, X, bias, out, M, N, K, xpacked, opacked, nwn, plane_rows);
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
                            int M, int N, int K, int splits, int xpacked, int opacked, int plane_rows, hipStream_t st) {
  const int KB = K / 32;
  const int groups = N / (16 * C);
  if (epi == EPI_PART32) {
    // 3-4 row tiles, a long K per split and enough feature groups: 4 columns of 2 wavefronts
    // (64 rows, 8192 x 28672, 8 splits: 96 -> 87 us)
    if constexpr (MT >= 3 && C == 4)
      if (groups % 4 == 0 && groups / 4 * splits >= 200 && KB / splits >= 64)
        return launch_w<T, MT, C, 8, true>(epi, 8, 4, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
    // 3-4 row tiles otherwise: 8 wavefronts (few splits, see gemm_skinny_splits); up to 2 row tiles:
    // 4 wavefronts, the K split across workgroups provides the parallelism
    if constexpr (MT >= 3)
      return launch_w<T, MT, C, 8, false>(epi, 8, 1, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
    else
      return launch_w<T, MT, C, 16, false>(epi, (MT == 1 && splits == 1) ? 8 : 4, 1, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
  }
  if constexpr (MT >= 3) {      // 8 wavefronts at most: twice the registers, nothing spills
    const int nwn = pick_columns(MT, groups, KB, 8);
    if (nwn > 1) return launch_w<T, MT, C, 8, true>(epi, 8, nwn, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
    return launch_w<T, MT, C, 8, false>(epi, 8, 1, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
  } else {
    const int ks = pick_ks(groups, KB);
    const int nwn = pick_columns(MT, groups, KB, ks);
    if (nwn > 1) return launch_w<T, MT, C, 16, true>(epi, ks, nwn, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
    return launch_w<T, MT, C, 16, false>(epi, ks, 1, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
  }
}

// Column blocks per wavefront: as many as row tiles (activation traffic <= weight
// traffic), limited by what divides the number of 16-row weight blocks; SwiGLU needs
// an even count (gate/up pairs).
template <class T>
static hipError_t launch_t(int epi, const uint16_t* W, const uint16_t* X, const uint16_t* bias, void* out, int M,
                           int N, int K, int splits, int xpacked, int opacked, int plane_rows, hipStream_t st) {
  const int nb = N / 16;
  const bool dual = epi == EPI_SWIGLU16;
  if (M > 64) {
    // 65..128 rows.  Packed activations and enough feature groups: the LDS-sharing kernel with 6 or 8 row tiles and
    // two column blocks per wavefront (the weights still cross the chip once).  Otherwise two passes of up to 64 rows
    // (the weights are read twice: only shapes with few feature groups or row-major activations get here).
    if (xpacked && epi != EPI_RESID32 && nb % 2 == 0) {
      WidePlan pl{2, 4, 8};
      bool ok;
      if (epi == EPI_PART32) {
        const SplitPlan sp = plan_split(M, nb, K / 32);
        const int groups = nb / 2;
        if (sp.splits == splits) {       // the planned number of planes: the planned shape
          ok = true;
          pl = WidePlan{2, sp.nwn, sp.nwn};
        } else {
          ok = groups % 4 == 0 && groups / 4 * splits >= 200 && (K / 32) / splits >= 64;
        }
      } else {
        pl = plan_wide(nb, K / 32, 2);
        ok = pl.nwn >= 4;
      }
      if (ok) {
        if (M <= 96) return launch_wide<T, 6, 2>(epi, pl.ks, pl.nwn, W, X, bias, out, M, N, K, splits, opacked, plane_rows, st);
        return launch_wide<T, 8, 2>(epi, pl.ks, pl.nwn, W, X, bias, out, M, N, K, splits, opacked, plane_rows, st);
      }
    }
    const hipError_t e = launch_t<T>(epi, W, X, bias, out, 64, N, K, splits, xpacked, opacked, plane_rows, st);
    if (e != hipSuccess) return e;
    const int ncols = dual ? N / 2 : N;
    const uint16_t* X2 = X + (size_t)64 * K;                    // 4 row tiles further on, packed or row-major
    void* out2 = (epi == EPI_PART32 || epi == EPI_RESID32) ? static_cast<void*>(static_cast<float*>(out) + (size_t)64 * ncols)
                                                           : static_cast<void*>(static_cast<uint16_t*>(out) + (size_t)64 * ncols);
    return launch_t<T>(epi, W, X2, bias, out2, M - 64, N, K, splits, xpacked, opacked, plane_rows, st);
  }
  // Up to 8 rows: the burst kernel (the LDS-sharing one measured 5 % slower at K = 4096 and 1-6 % faster at
  // K = 7168).  9..16 rows: it loads all 16 rows of a tile and slows down (21504 x 7168: 50 -> 57 us), the
  // LDS-sharing kernel does not (48 us).
  if (M <= 8 || (M <= 16 && !(xpacked && epi != EPI_RESID32))) {
    if (dual) return launch_mc<T, 1, 2>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
    return launch_mc<T, 1, 1>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
  }
  if (xpacked && epi != EPI_RESID32) {
    // 9..64 rows, packed activations: the kernel that shares them through LDS, where a launch shape exists
    WidePlan pl{0, 1, 8};
    bool ok;
    if (epi == EPI_PART32) {
      // split-K planes: the planned shape when the caller asks for the planned number of planes
      // (gemm_skinny_splits); for any other number, 4 columns of 2 wavefronts, 4 column blocks each, where
      // the feature groups times the splits fill the chip and every split keeps a long K
      const SplitPlan sp = plan_split(M, nb, K / 32);
      const int groups = nb / 4;
      if (sp.splits == splits) {
        ok = true;
        pl = WidePlan{sp.C, sp.nwn, sp.nwn};
      } else {
        ok = nb % 4 == 0 && groups % 4 == 0 && groups / 4 * splits >= 200 && (K / 32) / splits >= 64;
        pl = WidePlan{4, 4, 8};
      }
    } else {
      pl = plan_wide(nb, K / 32);
      ok = pl.nwn >= 4;
    }
    if (ok && !(dual && pl.C % 2)) {
      if (M <= 16) {
        if (pl.C == 4) return launch_wide<T, 1, 4>(epi, pl.ks, pl.nwn, W, X, bias, out, M, N, K, splits, opacked, plane_rows, st);
        return launch_wide<T, 1, 2>(epi, pl.ks, pl.nwn, W, X, bias, out, M, N, K, splits, opacked, plane_rows, st);
      }
      if (M <= 32) {
        if (pl.C == 4) return launch_wide<T, 2, 4>(epi, pl.ks, pl.nwn, W, X, bias, out, M, N, K, splits, opacked, plane_rows, st);
        return launch_wide<T, 2, 2>(epi, pl.ks, pl.nwn, W, X, bias, out, M, N, K, splits, opacked, plane_rows, st);
      }
      if (M <= 48) {
        if (pl.C == 4) return launch_wide<T, 3, 4>(epi, pl.ks, pl.nwn, W, X, bias, out, M, N, K, splits, opacked, plane_rows, st);
        return launch_wide<T, 3, 2>(epi, pl.ks, pl.nwn, W, X, bias, out, M, N, K, splits, opacked, plane_rows, st);
      }
      if (pl.C == 4) return launch_wide<T, 4, 4>(epi, pl.ks, pl.nwn, W, X, bias, out, M, N, K, splits, opacked, plane_rows, st);
      return launch_wide<T, 4, 2>(epi, pl.ks, pl.nwn, W, X, bias, out, M, N, K, splits, opacked, plane_rows, st);
    }
  }
  if (M <= 16) {
    if (dual) return launch_mc<T, 1, 2>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
    return launch_mc<T, 1, 1>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
  }
  if (M <= 32) {
    if (nb % 2 == 0) return launch_mc<T, 2, 2>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
    return launch_mc<T, 2, 1>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
  }
  if (M <= 48) {
    if (nb % 4 == 0) return launch_mc<T, 3, 4>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
    if (nb % 2 == 0) return launch_mc<T, 3, 2>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
    return launch_mc<T, 3, 1>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
  }
  if (nb % 4 == 0) return launch_mc<T, 4, 4>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
  if (nb % 2 == 0) return launch_mc<T, 4, 2>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
  return launch_mc<T, 4, 1>(epi, W, X, bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
}

hipError_t launch_gemm_skinny(int dtype, int epi, const void* W, const void* X, const void* bias, void* out,
                              int M, int N, int K, hipStream_t st, int splits, int flags) {
  const int xpacked = flags & kXPacked ? 1 : 0, opacked = flags & kOutPacked ? 1 : 0;
  if (opacked && (epi == EPI_RESID32 || epi == EPI_PART32)) return hipErrorInvalidValue;
  if (opacked && (epi == EPI_SWIGLU16 ? (N / 2) % 32 : N % 32)) return hipErrorInvalidValue;
  if (M <= 0) return hipSuccess;
  if (M > kMaxDecodeRows || N % 16 || K % 32 || (epi == EPI_SWIGLU16 && N % 32)) return hipErrorInvalidValue;
  if (epi == EPI_PART32 ? (splits < 1 || splits > kMaxSplits) : splits != 1) return hipErrorInvalidValue;
  const int plane_rows = M;                                    // rows of one plane of partial sums
  if (dtype == 0)
    return launch_t<F16>(epi, (const uint16_t*)W, (const uint16_t*)X, (const uint16_t*)bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
  return launch_t<BF16>(epi, (const uint16_t*)W, (const uint16_t*)X, (const uint16_t*)bias, out, M, N, K, splits, xpacked, opacked, plane_rows, st);
}

// Split count for the residual projections of a decode step (few output features, long
// K).  Up to 32 rows: enough 256-thread workgroups that every CU holds several, each
// wavefront still streaming at least 4 KiB of weights.  Above 32 rows every split costs a
// plane of 64 x N partial sums, written here and read again by the fold, so: 8 splits where
// the 4-column instance applies (long K, see launch_mc), else as few as give about one
// workgroup per CU (64 rows, 8192 x 8192: 2 splits 30.7 us, 8 splits 33.5 us).
int gemm_skinny_splits(int M, int N, int K) {
  const int KB = K / 32;
  if (M > 64) {
    // 6 or 8 row tiles: the planned shape where one exists; every other shape runs as two passes of up to 64 rows
    // and wants the split of 64 rows
    if (N % 16 == 0) {
      const SplitPlan pl = plan_split(M, N / 16, KB);
      if (pl.splits) return pl.splits;
    }
    return gemm_skinny_splits(64, N, K);
  }
  if (M > 8 && N % 16 == 0) {
    const SplitPlan pl = plan_split(M, N / 16, KB);
    if (pl.splits) return pl.splits;
  }
  const int C = M <= 16 ? 1 : (M <= 32 ? 2 : 4);
  const int groups = N / (16 * C);
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

// The QKV projection of a decode step at 9..128 rows: N = (Hq + 2 Hkv) d features are 160-1344 blocks, so the
// 16-bit-epilogue kernels run 120-170 workgroups (64 rows, 10240 x 8192: 46 us = 3.6 TB/s; 21504 x 7168: 78 us;
// 32 rows, 15360 x 5120: 30 us); split over K with the planned shape they fill the chip (30, 52, 28 us).
int gemm_qkv_splits(int M, int N, int K) {
  if (M <= 8 || M > kMaxDecodeRows || N % 16 || K % 32) return 0;
  const SplitPlan pl = plan_split(M, N / 16, K / 32);
  return pl.splits >= 2 ? pl.splits : 0;
}

}  // namespace sn
