// Prefill-phase projection: out = epilogue(X[M][K] * W^T) for many token rows.
//
// Prefill is the computation-intensive phase (paper Sec. 2.1): a dense contraction, so
// it runs on the matrix cores (v_mfma_f32_16x16x32, fp32 accumulate).  Weight tiles
// (16 features x 32 k) are stored in matrix-core lane order and are read straight from
// global memory into registers as the A operand (one coalesced 1 KiB request per tile);
// D[feature][token]: a lane ends up with 4 consecutive features of one token, which
// makes the row-major output store a short vector.
//
// Three kernels:
//  * gemm_tile_big_kernel (further down) -- N % 256 == 0, K % 256 == 0 and more than 128 token rows: 256 tokens x 256
//    features per workgroup, one wavefront per SIMD; every full-size prefill runs on it.
//  * gemm_tile_lds_kernel -- N % 256 == 0, K % 64 == 0, whatever the first does not take.  A 256-thread
//    workgroup computes 128 tokens x 256 features; each wavefront owns 128 x 64 of it
//    (32 accumulator tiles).  The activation slab (128 tokens x 64 k) is shared by the
//    four wavefronts, so it is staged through LDS, double-buffered, already permuted
//    into B-operand lane order (conflict-free 16-byte reads); weights are private to a
//    wavefront, so they bypass LDS and are double-buffered in registers.  Workgroups
//    are numbered so that the ones resident on one XCD at a time share weight columns
//    and token rows in that XCD's L2.
//  * gemm_tile_kernel -- any N % 16 == 0, K % 32 == 0: 128 x 128 per workgroup, both
//    operands read directly from global memory.
#include <algorithm>

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
// Workgroup id -> output tile, XCD-aware.  Hardware deals consecutive workgroup ids round-robin to the 8 XCDs, each
// with its own L2.  An XCD gets a contiguous band of NT/8 feature tiles and walks it in groups of CB feature tiles:
// inside a group, token tile by token tile.  The ~32 workgroups an XCD runs at once are then about 32/CB token
// tiles x CB feature tiles: the CB workgroups of a token tile share its activations in that L2, the token tiles of
// a group share its weights, and only the weights of the 8 groups in progress are live in the memory-side cache
// (a group as wide as the whole band streams the band's weights once per token tile when they exceed that cache:
// 57344 x 8192 re-read 683 times at 131072 rows).
__device__ __forceinline__ void tile_of(int id, int NT, int TT, int CB, int& tn, int& tt) {
  if (NT % 8 == 0) {
    const int xcd = id & 7, j = id >> 3, band = NT >> 3;
    const int per_group = TT * CB;               // CB divides band
    const int gi = j / per_group, r = j % per_group;
    tt = r / CB;
    tn = xcd * band + gi * CB + r % CB;
  } else {
    tn = id % NT;
    tt = id / NT;
  }
}

// Feature tiles per group for tile_of in the 256 x 256 kernel.  An XCD runs about 32 workgroups at once: 32/d token tiles
// x d feature tiles, which fetch (32/d) x 256 + d x 256 operand rows per k step between them; the divisor d of the band
// that makes this smallest wins, whether or not the weights of the 8 groups then fit the memory-side cache.  Measured
// (with 192-token tiles) at 131072 rows: 57344 x 8192 (band 28) d = 4: 106 ms, 7: 107, 2: 109, 14: 112, 1: 120, 28: 128;
// 8192 x 28672 (band 4) d = 4: 52.3, 2: 54.1, 1: 60.0; 10240 x 8192 (band 5) d = 5: 19.0, 1: 20.0.
static int tile_group(int NT) {
  if (NT % 8) return 1;
  const int band = NT / 8;
  int cb = 1;
  long best = 32 * 256 + 256;
  for (int d = 2; d <= band && d <= 32; ++d) {
    const long rows = (32l * 256 + d - 1) / d + 256l * d;
    if (band % d == 0 && rows < best) best = rows, cb = d;
  }
  return cb;
}

// The 128 x 256 kernel (two workgroups per CU) keeps the rule it was tuned with: the
// largest divisor of the band whose 8 groups' weights fit half the memory-side cache, but two where the band allows it.
static int tile_group_lds(int NT, int K) {
  if (NT % 8) return 1;
  const int band = NT / 8;
  const long most = std::max(2l, (128l << 20) / (8l * 256 * K * 2));
  int cb = 1;
  for (int d = 1; d <= band; ++d)
    if (band % d == 0 && d <= most) cb = d;
  return cb;
}

template <class T, int EPI>
__global__ __launch_bounds__(256, 2) void gemm_tile_lds_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ X, const uint16_t* __restrict__ bias,
    void* __restrict__ out, int M, int N, int K, int NT, int TT, int CB) {
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
  tile_of(blockIdx.x, NT, TT, CB, tn, tt);
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
  // this lane's bias values depend on the feature block only: fetched once, not once per element
  // (128 two-byte loads per lane in the epilogue cost more than the stores)
  float bv[4][4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int n = EPI == EPI_SWIGLU16 ? ((nb0 + (j & ~1)) >> 1) * 16 + nl + ((j & 1) ? (N >> 1) : 0) : (nb0 + j) * 16 + nl;
    u16x4 b4 = u16x4{0, 0, 0, 0};
    if (bias) b4 = *reinterpret_cast<const u16x4*>(bias + n);
#pragma unroll
    for (int r = 0; r < 4; ++r) bv[j][r] = bias ? to_f32<T>(b4[r]) : 0.f;
  }
  if (EPI == EPI_RESID32) {
    // fp32 read-modify-write of the residual stream: all reads of a feature block are requested before
    // the first is used
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = (nb0 + j) * 16 + nl;
      f32x4 r[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int t = t0 + i * 16 + (lane & 15);
        r[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (t < M) r[i] = *reinterpret_cast<const f32x4*>(static_cast<float*>(out) + (size_t)t * N + n);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int t = t0 + i * 16 + (lane & 15);
#pragma unroll
        for (int q = 0; q < 4; ++q) r[i][q] += acc[j][i][q] + bv[j][q];
        if (t < M) *reinterpret_cast<f32x4*>(static_cast<float*>(out) + (size_t)t * N + n) = r[i];
      }
    }
    return;
  }
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
        for (int r = 0; r < 4; ++r) o[r] = from_f32<T>(silu(acc[j][i][r] + bv[j][r]) * (acc[j + 1][i][r] + bv[j + 1][r]));
        *reinterpret_cast<u16x4*>(static_cast<uint16_t*>(out) + (size_t)t * F + n) = o;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int n = (nb0 + j) * 16 + nl;
        u16x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float v = acc[j][i][q] + bv[j][q];
          if (EPI == EPI_GELU16) v = gelu_erf(v);
          o[q] = from_f32<T>(v);
        }
        *reinterpret_cast<u16x4*>(static_cast<uint16_t*>(out) + (size_t)t * N + n) = o;
      }
    }
  }
}


// ---------------------------------------------------------------------------------
// main path: 256 tokens x 256 features per workgroup, 256 x 64 per wavefront
// ---------------------------------------------------------------------------------
// One workgroup (4 wavefronts, one per SIMD, 512 registers each) per CU; a wavefront keeps 4 x 16
// accumulator tiles: 64 features x all 256 tokens, 64 MFMAs per 32-wide k step for 4 weight fragments of
// its own and 16 activation fragments from LDS (128 flop per byte fetched, against 87 for 128 x 256; with 4 x 12
// tiles, 192 tokens and 112 flop per byte, the same kernel measured 2-7 % slower: what a step costs beyond its
// MFMAs is the time its bytes take through the CU's one vector-memory path).
//   * weights of step t: global -> register set t % 4, requested three steps ahead (no weight is
//     fetched twice by a workgroup, none passes through LDS);
//   * activations of step t: global -> LDS buffer t % NB directly (global_load_lds_dwordx4: lane l's
//     16 bytes land at M0 + 16 l, which is exactly the B-operand tile order when lane l asks for
//     token l % 16, k chunk l / 16), requested NB - 1 steps ahead, no registers involved; each fragment
//     is re-read from LDS for the next step right after the four MFMAs that used it.
// What makes a lone wavefront per SIMD work (each found by measurement):
//   * memory requests are spread over the step -- one request, four MFMAs, one LDS read, and so on --
//     because a wavefront that queues its seven requests at once stalls behind them and nothing else
//     feeds its matrix core (1450 -> 1150 clocks per step of 48 MFMAs, measured with 192-token tiles);
//   * the direct-to-LDS loads are inline assembly, so that the compiler does not serialise every LDS
//     read behind the newest of them; their completion is awaited by hand: loads complete in issue
//     order, each step issues 4 of them and 4 weight loads per wavefront, so "the activations
//     of step t + 2 have landed" is s_waitcnt vmcnt(4 + 8 * (NB - 3)) at the end of step t (every
//     step issues its 8 requests, the last ones redundantly, so the count always holds).  The waits the
//     compiler inserts for the weight registers count only its own loads and therefore wait for more
//     than necessary -- never for less;
//   * the MFMAs are inline assembly with the accumulator tied to its registers (see mma_inplace);
//   * a bare s_barrier per step (no fence): it publishes the loads just awaited, and the buffer the
//     next step overwrites was read two steps ago;
//   * the epilogue fetches its bias values once per feature block (not per element: 20 -> 4 us per
//     tile), transposes the tile through the idle operand ring and stores whole cache lines, and for
//     the fp32 residual stream requests all its reads before using the first;
//   * all workgroups start together.  (While the epilogue still stored partial lines, starting the first workgroup of
//     each CU up to 3/4 of a tile late spread the epilogues' bursts and gained 20 % on one shape; with the present
//     epilogue the same stagger costs 1-7 % at many rounds of tiles and up to 30 % at three, so it is gone.)
// Ring indices must be compile-time constants, hence the k loop is unrolled by the ring depth, which
// must divide the number of k steps.  Token rows past M fetch row 0 and are never stored.
// Measured at 32768 rows (MI355X): 1.09-1.23 PFLOP/s against 0.86-0.99 for the kernel above; at 4096 rows
// (12288 x 4096: 768 tiles, three rounds of one workgroup per CU) 0.32 ms against 0.52-0.56 ms, at 1024 rows
// (4096 x 16384: 64 tiles) 0.29 against 0.39 ms.  It takes every shape with more than one 128-row tile of tokens
// (below that half of its 256-token tile would be idle arithmetic) whose N and K are multiples of 256.
constexpr int kBigTileMinRows = 129;
constexpr int kBigTileRing = 8;          // LDS buffers / weight register sets of the 256 x 256 kernel (look-ahead 7 k steps)
constexpr int kBigTileWeightRing = 4;    // weight register sets of the 256 x 256 kernel (look-ahead 3 k steps)
constexpr int kBigTileTokenTiles = 16;  // 16-token tiles per workgroup (256 tokens): 4 x 16 accumulator tiles per wavefront

template <int V>
struct IC {
  static constexpr int value = V;
};

// In-place MFMA (accumulator tied to its registers).  With the builtin, the register allocator gives a
// loop-carried accumulator different registers at the top and at the bottom of the unrolled k loop and
// repairs that with ~190 accumulator moves per trip; a tied operand leaves it no such freedom.  The compiler
// cannot see inside: operands come from loads (it still inserts their waits), an accumulator is touched once
// per k step (48 MFMAs apart), and the accumulators are first read long after the last MFMA (a counter
// wait, a barrier and the bias loads come first), so no matrix-core hazard needs a hand-placed wait state.
template <class T>
__device__ __forceinline__ void mma_inplace(f32x4& c, const u16x8& a, const u16x8& b);
template <>
__device__ __forceinline__ void mma_inplace<F16>(f32x4& c, const u16x8& a, const u16x8& b) {
  asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}
template <>
__device__ __forceinline__ void mma_inplace<BF16>(f32x4& c, const u16x8& a, const u16x8& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <class T, int EPI, int TI>   // TI: 16-token tiles per workgroup
__global__ __launch_bounds__(256, 1) void gemm_tile_big_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ X, const uint16_t* __restrict__ bias,
    void* __restrict__ out, int M, int N, int K, int NT, int TT, int CB, int xpacked, int opacked) {
  constexpr int BM = TI * 16;             // tokens per workgroup
  constexpr int XT = TI / 4;              // token tiles each wavefront stages per k step
  constexpr int FJ = 4;                   // 16-feature blocks per wavefront
  constexpr int NB = kBigTileRing;        // ring depth: LDS buffers and weight register sets
  constexpr int D = NB - 1;               // look-ahead in k steps
  constexpr int kTile = 64 * 8;           // elements of one 16 x 32 operand tile
  static_assert(XT + FJ <= TI && FJ == 4 && D >= 3 && D <= 7 && FJ + (XT + FJ) * (D - 2) < 64,
                "the hand-written wait counts XT + FJ loads per step in a 6-bit counter");
  __shared__ __attribute__((aligned(16))) uint16_t xs[NB][TI][kTile];   // 8 x 12 KiB

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int S = K >> 5;                      // k steps

  int tn, tt;                                // XCD-aware numbering, as in gemm_tile_lds_kernel
  tile_of(blockIdx.x, NT, TT, CB, tn, tt);
  const int t0 = tt * BM;
  const int nb0 = tn * 16 + wave * FJ;       // first of this wavefront's feature blocks
  const uint16_t* wp = W + ((size_t)nb0 * S) * 512 + lane * 8;
  const size_t wstride = (size_t)S * 512;

  // activation staging: wavefront w fetches token tiles XT*w .. XT*w + XT - 1 of the workgroup's TI
  // Row-major X: a lane's 16 bytes are k-chunk lane / 16 of token row lane % 16, 64 bytes per row and request.
  // Row-tile packed X (common.h packed_off): the tile of a k step is one contiguous KiB in exactly the order
  // the LDS stage wants, so a request reads 8 whole cache lines instead of 16 half ones.
  const uint16_t* xg[XT];
  const int xstep = xpacked ? kTile : 32;    // elements from one k step to the next
#pragma unroll
  for (int i = 0; i < XT; ++i) {
    const int row = t0 + (wave * XT + i) * 16 + (lane & 15);
    if (xpacked) {
      const int tile = (t0 >> 4) + wave * XT + i;
      xg[i] = X + (size_t)(tile * 16 < M ? tile : 0) * S * kTile + lane * 8;
    } else {
      xg[i] = X + (size_t)(row < M ? row : 0) * K + (lane >> 4) * 8;
    }
  }
  // LDS byte address of this wavefront's first staging tile in buffer 0 (wave-uniform)
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)&xs[0][wave * XT][0]);

  f32x4 acc[FJ][TI];                         // [feature block][token tile]
#pragma unroll
  for (int j = 0; j < FJ; ++j)
#pragma unroll
    for (int i = 0; i < TI; ++i) acc[j][i] = f32x4{0.f, 0.f, 0.f, 0.f};

  constexpr int NW = kBigTileWeightRing;   // weight register sets (look-ahead NW - 1 steps)
  static_assert(NB % NW == 0, "the unrolled loop must bring both rings back to slot 0");
  u16x8 a[NW][FJ], bf[TI];
  auto load_w = [&](auto set, int st) __attribute__((always_inline)) {
    constexpr int R = decltype(set)::value;
#pragma unroll
    for (int j = 0; j < FJ; ++j) a[R][j] = *reinterpret_cast<const u16x8*>(wp + j * wstride + (size_t)st * 512);
  };
  auto dma_x = [&](auto buf, int st) __attribute__((always_inline)) {
    constexpr int B = decltype(buf)::value;
#pragma unroll
    for (int i = 0; i < XT; ++i) {
      const uint16_t* g = xg[i] + (size_t)st * xstep;
      const uint32_t m0 = lds0 + (uint32_t)((B * TI + i) * kTile * 2);
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(m0) : "memory");
    }
  };
  // k step st (st % NB == U)
  auto step = [&](auto uc, auto, int st) __attribute__((always_inline)) {
    constexpr int U = decltype(uc)::value;
    constexpr int R = (U + D) % NB;           // LDS ring slot being refilled
    constexpr int RW = (U + NW - 1) % NW;     // weight register set being refilled
    constexpr int BN = (U + 1) % NB;          // LDS buffer of the next step
    const int ahead = st + D < S ? st + D : S - 1;
    const int ahead_w = st + NW - 1 < S ? st + NW - 1 : S - 1;
    // One memory request, four MFMAs, one LDS read, twelve times over: a wavefront alone on its SIMD
    // must never sit in a queue of its own requests while the matrix core runs dry.
#pragma unroll
    for (int i = 0; i < TI; ++i) {
      if (i < XT) {
        const uint16_t* g = xg[i] + (size_t)ahead * xstep;
        const uint32_t m0 = lds0 + (uint32_t)((R * TI + i) * kTile * 2);
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(m0) : "memory");
      } else if (i < XT + FJ) {
        a[RW][i - XT] = *reinterpret_cast<const u16x8*>(wp + (i - XT) * wstride + (size_t)ahead_w * 512);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < FJ; ++j) mma_inplace<T>(acc[j][i], a[U % NW][j], bf[i]);
      __builtin_amdgcn_sched_barrier(0);
      bf[i] = *reinterpret_cast<const u16x8*>(&xs[BN][i][lane * 8]);   // next step's fragment; after the last step: stale, unused
      __builtin_amdgcn_sched_barrier(0);
    }
    wait_vmcnt<FJ + (XT + FJ) * (D - 2)>();   // this wavefront's share of the activations of step st + 2 has landed
    // Bare barrier (no fence): what it publishes are the direct-to-LDS loads just awaited, and the buffer
    // the next step overwrites was read into registers two steps ago.  A fence would also wait for the
    // fragment reads issued a moment ago, which are not needed before the next step.
    asm volatile("s_barrier" ::: "memory");
  };

  // prologue: the first seven steps' operands, all awaited (one exposed latency per tile)
  auto prologue = [&](auto uc) __attribute__((always_inline)) {
    constexpr int U = decltype(uc)::value;
    if (U < D) dma_x(IC<U>{}, U);
    if (U < NW - 1) load_w(IC<U % NW>{}, U);
  };
  prologue(IC<0>{});
  prologue(IC<1>{});
  prologue(IC<2>{});
  if (D > 3) prologue(IC<3 % NB>{});
  if (D > 4) prologue(IC<4 % NB>{});
  if (D > 5) prologue(IC<5 % NB>{});
  if (D > 6) prologue(IC<6 % NB>{});
  wait_vmcnt<0>();
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TI; ++i) bf[i] = *reinterpret_cast<const u16x8*>(&xs[0][i][lane * 8]);

  // S is a multiple of NB (the launcher sees to it).  Every step requests operands without a condition --
  // the last D steps re-request the final step's (harmless: those ring slots are free) -- because the
  // compiler's own waits for the weight registers are only as tight as what it knows was requested since.
  for (int s = 0; s < S; s += NB) {
    step(IC<0>{}, IC<1>{}, s);
    step(IC<1>{}, IC<1>{}, s + 1);
    step(IC<2>{}, IC<1>{}, s + 2);
    step(IC<3>{}, IC<1>{}, s + 3);
    if (NB > 4) step(IC<4 % NB>{}, IC<1>{}, s + 4);
    if (NB > 5) step(IC<5 % NB>{}, IC<1>{}, s + 5);
    if (NB > 6) step(IC<6 % NB>{}, IC<1>{}, s + 6);
    if (NB > 7) step(IC<7 % NB>{}, IC<1>{}, s + 7);
  }
  wait_vmcnt<0>();   // the redundant requests of the last steps

  const int nl = (lane >> 4) * 4;
  if (EPI == EPI_RESID32) {
    // fp32 read-modify-write of the residual stream, through the idle operand ring as well (see below):
    // two halves of 128 tokens x 256 features x 4 bytes; 16-byte chunks swizzled by chunk ^ (token % 16);
    // afterwards every thread adds 16 contiguous bytes into the stream, a token's 1 KiB row as whole lines.
    static_assert(TI % 2 == 0 && (TI / 2) * 16 * 256 * 4 <= NB * TI * kTile * 2, "half the fp32 tile must fit the ring");
    float* fb = reinterpret_cast<float*>(&xs[0][0][0]);
    float bvr[FJ][4];
#pragma unroll
    for (int j = 0; j < FJ; ++j) {
      u16x4 b4 = u16x4{0, 0, 0, 0};
      if (bias) b4 = *reinterpret_cast<const u16x4*>(bias + (nb0 + j) * 16 + nl);
#pragma unroll
      for (int r = 0; r < 4; ++r) bvr[j][r] = bias ? to_f32<T>(b4[r]) : 0.f;
    }
    const int q = threadIdx.x & 63, r0 = threadIdx.x >> 6;       // 16-byte chunk of the row, first row of this thread
    float* xg0 = static_cast<float*>(out) + (size_t)tn * 256 + q * 4;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      __syncthreads();                                            // ring (or the previous half) no longer read
#pragma unroll
      for (int ii = 0; ii < TI / 2; ++ii) {
        const int i = h * (TI / 2) + ii;
        const int tok = ii * 16 + (lane & 15);
#pragma unroll
        for (int j = 0; j < FJ; ++j) {
          f32x4 v = acc[j][i];
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] += bvr[j][r];
          const int c = wave * 16 + j * 4 + (lane >> 4);
          *reinterpret_cast<f32x4*>(fb + (size_t)tok * 256 + ((c ^ (lane & 15)) << 2)) = v;
        }
      }
      __syncthreads();
      // all of this thread's stream reads are requested before the first is used (one latency, not 24)
      constexpr int ROWS = (TI / 2) * 16 / 4;
      f32x4 r[ROWS];
#pragma unroll
      for (int k = 0; k < ROWS; ++k) {
        const int t = t0 + h * (TI / 2) * 16 + r0 + 4 * k;
        r[k] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (t < M) r[k] = *reinterpret_cast<const f32x4*>(xg0 + (size_t)t * N);
      }
#pragma unroll
      for (int k = 0; k < ROWS; ++k) {
        const int tok = r0 + 4 * k;
        const int t = t0 + h * (TI / 2) * 16 + tok;
        r[k] += *reinterpret_cast<const f32x4*>(fb + (size_t)tok * 256 + ((q ^ (tok & 15)) << 2));
        if (t < M) *reinterpret_cast<f32x4*>(xg0 + (size_t)t * N) = r[k];
      }
    }
    return;
  }
  // 16-bit outputs.  A lane holds 4 consecutive features of one token per accumulator tile, so a direct
  // store writes 32-byte pieces of cache lines (measured: ~20 us per tile, a quarter of the kernel).  The
  // tile is therefore transposed through the now idle operand ring: [256 tokens][OW features], 8-byte chunks
  // swizzled by chunk ^ (token % 16) so that the 16 tokens a store instruction covers hit 16 different
  // bank pairs; then every thread moves 16 contiguous bytes and a token's row leaves as whole lines.
  constexpr bool DUAL = EPI == EPI_SWIGLU16;
  constexpr int OW = DUAL ? 128 : 256;                 // output features of this workgroup
  static_assert(TI * 16 * OW * 2 <= NB * TI * kTile * 2, "output tile must fit the operand ring");
  uint16_t* ob = &xs[0][0][0];
  // this lane's bias values, fetched once (they depend on the feature block only, not on the token tile)
  float bv[FJ][4];
#pragma unroll
  for (int j = 0; j < FJ; ++j) {
    const int F = N >> 1;
    const int n = DUAL ? ((nb0 + (j & ~1)) >> 1) * 16 + nl + ((j & 1) ? F : 0) : (nb0 + j) * 16 + nl;
    u16x4 b4 = u16x4{0, 0, 0, 0};
    if (bias) b4 = *reinterpret_cast<const u16x4*>(bias + n);
#pragma unroll
    for (int r = 0; r < 4; ++r) bv[j][r] = bias ? to_f32<T>(b4[r]) : 0.f;
  }
  __syncthreads();                                     // every wavefront is done with the ring
#pragma unroll
  for (int i = 0; i < TI; ++i) {
    const int tok = i * 16 + (lane & 15);
#pragma unroll
    for (int j = 0; j < FJ; j += (DUAL ? 2 : 1)) {
      u16x4 o;
      if (DUAL) {
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = from_f32<T>(silu(acc[j][i][r] + bv[j][r]) * (acc[j + 1][i][r] + bv[j + 1][r]));
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float v = acc[j][i][r] + bv[j][r];
          if (EPI == EPI_GELU16) v = gelu_erf(v);
          o[r] = from_f32<T>(v);
        }
      }
      const int c = DUAL ? wave * 8 + (j >> 1) * 4 + (lane >> 4) : wave * 16 + j * 4 + (lane >> 4);   // 8-byte chunk in the row
      *reinterpret_cast<u16x4*>(ob + (size_t)tok * OW + ((c ^ (lane & 15)) << 2)) = o;
    }
  }
  __syncthreads();
  constexpr int PIECES = OW / 8;                       // 16-byte pieces per token row
  constexpr int RPP = 256 / PIECES;                    // token rows per pass of the workgroup
  const int ON = DUAL ? N >> 1 : N;
  if (opacked) {
    // row-tile packed output (it feeds another projection): a wavefront writes one 16-token x 32-feature tile,
    // 1 KiB contiguous, per pass -- lane = token % 16 + 16 * (16-byte piece of the tile)
    constexpr int PT = PIECES / 4;                     // 32-feature tiles across the workgroup's features
    uint16_t* og = static_cast<uint16_t*>(out);
    const int tk = lane & 15, pc = lane >> 4;
#pragma unroll 4
    for (int tix = wave; tix < TI * PT; tix += 4) {
      const int tok = (tix / PT) * 16 + tk, q = (tix % PT) * 4 + pc;
      u16x8 v = *reinterpret_cast<const u16x8*>(ob + (size_t)tok * OW + ((q ^ (tk >> 1)) << 3));
      if (tk & 1) v = u16x8{v[4], v[5], v[6], v[7], v[0], v[1], v[2], v[3]};
      if (t0 + tok < M) *reinterpret_cast<u16x8*>(og + packed_off(t0 + tok, tn * OW + q * 8, ON >> 5)) = v;
    }
    return;
  }
  const int q = threadIdx.x % PIECES, r0 = threadIdx.x / PIECES;
  uint16_t* og = static_cast<uint16_t*>(out) + (size_t)tn * OW + q * 8;
#pragma unroll 4
  for (int tok = r0; tok < BM; tok += RPP) {
    const int t = tok & 15;
    u16x8 v = *reinterpret_cast<const u16x8*>(ob + (size_t)tok * OW + ((q ^ (t >> 1)) << 3));
    if (t & 1) v = u16x8{v[4], v[5], v[6], v[7], v[0], v[1], v[2], v[3]};
    if (t0 + tok < M) *reinterpret_cast<u16x8*>(og + (size_t)(t0 + tok) * ON) = v;
  }
}

template <class T>
static hipError_t launch_t(int epi, const uint16_t* W, const uint16_t* X, const uint16_t* bias, void* out, int M,
                           int N, int K, int xpacked, int opacked, hipStream_t st) {
  constexpr int TI = kBigTileTokenTiles;
  if (N % 256 == 0 && K % (32 * kBigTileRing) == 0 && M >= kBigTileMinRows) {
    const int NT = N / 256, TT = (M + TI * 16 - 1) / (TI * 16), CB = tile_group(NT);
    dim3 grid(NT * TT), block(256);
    switch (epi) {
      case EPI_STORE16:
        SN_LAUNCH((gemm_tile_big_kernel<T, EPI_STORE16, TI>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT, CB, xpacked, opacked);
        break;
      case EPI_GELU16:
        SN_LAUNCH((gemm_tile_big_kernel<T, EPI_GELU16, TI>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT, CB, xpacked, opacked);
        break;
      case EPI_RESID32:
        SN_LAUNCH((gemm_tile_big_kernel<T, EPI_RESID32, TI>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT, CB, xpacked, opacked);
        break;
      case EPI_SWIGLU16:
        SN_LAUNCH((gemm_tile_big_kernel<T, EPI_SWIGLU16, TI>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT, CB, xpacked, opacked);
        break;
      default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  if (xpacked || opacked) return hipErrorInvalidValue;
  if (N % 256 == 0 && K % 64 == 0) {
    const int NT = N / 256, TT = (M + 127) / 128, CB = tile_group_lds(NT, K);
    dim3 grid(NT * TT), block(256);
    switch (epi) {
      case EPI_STORE16:
        SN_LAUNCH((gemm_tile_lds_kernel<T, EPI_STORE16>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT, CB);
        break;
      case EPI_GELU16:
        SN_LAUNCH((gemm_tile_lds_kernel<T, EPI_GELU16>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT, CB);
        break;
      case EPI_RESID32:
        SN_LAUNCH((gemm_tile_lds_kernel<T, EPI_RESID32>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT, CB);
        break;
      case EPI_SWIGLU16:
        SN_LAUNCH((gemm_tile_lds_kernel<T, EPI_SWIGLU16>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT, CB);
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
                            int N, int K, hipStream_t st, int flags) {
  if (M <= 0) return hipSuccess;
  if (N % 16 || K % 32 || (epi == EPI_SWIGLU16 && N % 32)) return hipErrorInvalidValue;
  const int xpacked = flags & kXPacked ? 1 : 0, opacked = flags & kOutPacked ? 1 : 0;
  if (opacked && (epi == EPI_RESID32 || (epi == EPI_SWIGLU16 ? (N / 2) % 32 : N % 32))) return hipErrorInvalidValue;
  if (dtype == 0)
    return launch_t<F16>(epi, (const uint16_t*)W, (const uint16_t*)X, (const uint16_t*)bias, out, M, N, K, xpacked, opacked, st);
  return launch_t<BF16>(epi, (const uint16_t*)W, (const uint16_t*)X, (const uint16_t*)bias, out, M, N, K, xpacked, opacked, st);
}

// Whether launch_gemm_tile would run this shape on the 256 x 256 kernel, the one that reads and writes row-tile
// packed activations.
bool gemm_tile_takes_packed(int M, int N, int K) {
  return N % 256 == 0 && K % (32 * kBigTileRing) == 0 && M >= kBigTileMinRows;
}

}  // namespace sn
