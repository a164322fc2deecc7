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


// ---------------------------------------------------------------------------------
// large-M path: 192 tokens x 256 features per workgroup, 192 x 64 per wavefront
// ---------------------------------------------------------------------------------
// The 128 x 256 tile of the kernel above fetches 24 KiB per 2.1 MFLOP from the L2 (87 flop per
// byte) and, more to the point, keeps only ~64 KiB of requests in flight per CU: counters show
// its wavefronts (and those of any variant with a two-step look-ahead) waiting on memory 40 % of
// the time, because ~15 % of the L2 requests of a tile sweep miss (eight L2s, each re-reading
// the operands) and take well over a microsecond under load.  Hiding that at matrix-core speed
// needs ~150 KiB in flight per CU.  Here:
//   * workgroup tile 192 x 256 (112 flop per byte), one workgroup (4 wavefronts) per CU; a
//     wavefront keeps 4 x 12 accumulator tiles: 64 features x all 192 tokens, 48 MFMAs per
//     32-wide k step for 4 weight fragments of its own and 12 activation fragments from LDS;
//   * weights of step t: global -> register set t % NB, requested NB - 1 steps ahead (no weight
//     is fetched twice by a workgroup, none passes through LDS);
//   * activations of step t: global -> LDS buffer t % NB directly (global_load_lds_dwordx4:
//     lane l's 16 bytes land at M0 + 16 l, which is exactly the B-operand tile order when lane
//     l asks for token l % 16, k chunk l / 16), requested NB - 1 steps ahead, no registers
//     involved; fragments are read from LDS half a step before use (two sets of 6).
// The direct-to-LDS loads are inline assembly (so that the compiler does not serialise every
// LDS read behind the newest of them), hence their completion is awaited by hand: loads
// complete in issue order, each step issues 3 of them followed by 4 weight loads per
// wavefront, so "the activations of step t + 2 have landed" is s_waitcnt vmcnt(4 + 7 * (NB - 3)) at
// the end of step t (every step issues its 7 requests, the last ones redundantly).  The waits
// the compiler inserts for the weight registers count only its own loads and therefore wait
// for more than necessary -- never for less.  Ring indices must be compile-time constants,
// hence the k loop is unrolled by the ring depth, which must divide the number of k steps.
// Token rows past M fetch row 0 and are never stored.
// From this many token rows on the 192 x 256 workgroup tile is used (below it too much of a
// tile would be padding and too few workgroups would exist).
constexpr int kBigTileMinRows = 1024;
constexpr int kBigTileRing = 8;          // LDS buffers / weight register sets of the 192 x 256 kernel (look-ahead 7 k steps)
constexpr int kBigTileTokenTiles = 12;  // 16-token tiles per workgroup (192 tokens): 4 x 12 accumulator tiles per wavefront

template <int V>
struct IC {
  static constexpr int value = V;
};

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <class T, int EPI, int TI>   // TI: 16-token tiles per workgroup
__global__ __launch_bounds__(256, 1) void gemm_tile_big_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ X, const uint16_t* __restrict__ bias,
    void* __restrict__ out, int M, int N, int K, int NT, int TT) {
  constexpr int BM = TI * 16;             // tokens per workgroup
  constexpr int XT = TI / 4;              // token tiles each wavefront stages per k step
  constexpr int FJ = 4;                   // 16-feature blocks per wavefront
  constexpr int NB = kBigTileRing;        // ring depth: LDS buffers and weight register sets
  constexpr int D = NB - 1;               // look-ahead in k steps
  constexpr int HT = TI / 2;              // token tiles per fragment set
  constexpr int kTile = 64 * 8;           // elements of one 16 x 32 operand tile
  static_assert(XT == 3 && FJ == 4 && D >= 3 && D <= 7, "the hand-written wait counts 3 + 4 loads per step");
  __shared__ __attribute__((aligned(16))) uint16_t xs[NB][TI][kTile];   // 8 x 12 KiB

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int S = K >> 5;                      // k steps

  int tn, tt;                                // XCD-aware numbering, as in gemm_tile_lds_kernel
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
  const int nb0 = tn * 16 + wave * FJ;       // first of this wavefront's feature blocks
  const uint16_t* wp = W + ((size_t)nb0 * S) * 512 + lane * 8;
  const size_t wstride = (size_t)S * 512;

  // activation staging: wavefront w fetches token tiles XT*w .. XT*w + XT - 1 of the workgroup's TI
  const uint16_t* xg[XT];
#pragma unroll
  for (int i = 0; i < XT; ++i) {
    const int row = t0 + (wave * XT + i) * 16 + (lane & 15);
    xg[i] = X + (size_t)(row < M ? row : 0) * K + (lane >> 4) * 8;
  }
  // LDS byte address of this wavefront's first staging tile in buffer 0 (wave-uniform)
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)&xs[0][wave * XT][0]);

  f32x4 acc[FJ][TI];                         // [feature block][token tile]
#pragma unroll
  for (int j = 0; j < FJ; ++j)
#pragma unroll
    for (int i = 0; i < TI; ++i) acc[j][i] = f32x4{0.f, 0.f, 0.f, 0.f};

  u16x8 a[NB][FJ], bf[2][HT];
  auto load_w = [&](auto set, int st) __attribute__((always_inline)) {
    constexpr int R = decltype(set)::value;
#pragma unroll
    for (int j = 0; j < FJ; ++j) a[R][j] = *reinterpret_cast<const u16x8*>(wp + j * wstride + (size_t)st * 512);
  };
  auto dma_x = [&](auto buf, int st) __attribute__((always_inline)) {
    constexpr int B = decltype(buf)::value;
#pragma unroll
    for (int i = 0; i < XT; ++i) {
      const uint16_t* g = xg[i] + (size_t)st * 32;
      const uint32_t m0 = lds0 + (uint32_t)((B * TI + i) * kTile * 2);
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(m0) : "memory");
    }
  };
  auto read_b = [&](auto half, auto buf) __attribute__((always_inline)) {
    constexpr int H = decltype(half)::value, B = decltype(buf)::value;
#pragma unroll
    for (int i = 0; i < HT; ++i) bf[H][i] = *reinterpret_cast<const u16x8*>(&xs[B][H * HT + i][lane * 8]);
  };
  // k step st (st % NB == U)
  auto step = [&](auto uc, auto, int st) __attribute__((always_inline)) {
    constexpr int U = decltype(uc)::value;
    const int ahead = st + D < S ? st + D : S - 1;
    dma_x(IC<(U + D) % NB>{}, ahead);
    load_w(IC<(U + D) % NB>{}, ahead);
    __builtin_amdgcn_sched_barrier(0);   // requests leave before this step's arithmetic
#pragma unroll
    for (int i = 0; i < HT; ++i)
#pragma unroll
      for (int j = 0; j < FJ; ++j) acc[j][i] = mma16x16x32<T>(a[U][j], bf[0][i], acc[j][i]);
    __builtin_amdgcn_sched_barrier(0);
    read_b(IC<0>{}, IC<(U + 1) % NB>{});   // after the last step: a stale buffer, never used
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < HT; ++i)
#pragma unroll
      for (int j = 0; j < FJ; ++j) acc[j][HT + i] = mma16x16x32<T>(a[U][j], bf[1][i], acc[j][HT + i]);
    __builtin_amdgcn_sched_barrier(0);
    read_b(IC<1>{}, IC<(U + 1) % NB>{});
    wait_vmcnt<4 + 7 * (D - 2)>();         // this wavefront's share of the activations of step st + 2 has landed
    // Bare barrier (no fence): what it publishes are the direct-to-LDS loads just awaited, and the buffer
    // the next step overwrites was read into registers two steps ago.  A fence would also wait for the
    // fragment reads issued a moment ago, which are not needed before the middle of the next step.
    asm volatile("s_barrier" ::: "memory");
  };

  // prologue: the first seven steps' operands, all awaited (one exposed latency per tile)
  auto prologue = [&](auto uc) __attribute__((always_inline)) {
    constexpr int U = decltype(uc)::value;
    if (U < D) {
      dma_x(IC<U>{}, U);
      load_w(IC<U>{}, U);
    }
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
  read_b(IC<0>{}, IC<0>{});
  read_b(IC<1>{}, IC<0>{});

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
#pragma unroll
  for (int i = 0; i < TI; ++i) {
    const int t = t0 + i * 16 + (lane & 15);
    if (t >= M) continue;
    if (EPI == EPI_SWIGLU16) {
      const int F = N >> 1;
#pragma unroll
      for (int j = 0; j < FJ; j += 2) {
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
      for (int j = 0; j < FJ; ++j) {
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
  if (N % 256 == 0 && M >= kBigTileMinRows && K % (32 * kBigTileRing) == 0) {
    constexpr int TI = kBigTileTokenTiles;
    const int NT = N / 256, TT = (M + TI * 16 - 1) / (TI * 16);
    dim3 grid(NT * TT), block(256);
    switch (epi) {
      case EPI_STORE16:
        SN_LAUNCH((gemm_tile_big_kernel<T, EPI_STORE16, TI>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT);
        break;
      case EPI_GELU16:
        SN_LAUNCH((gemm_tile_big_kernel<T, EPI_GELU16, TI>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT);
        break;
      case EPI_RESID32:
        SN_LAUNCH((gemm_tile_big_kernel<T, EPI_RESID32, TI>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT);
        break;
      case EPI_SWIGLU16:
        SN_LAUNCH((gemm_tile_big_kernel<T, EPI_SWIGLU16, TI>), grid, block, 0, st, W, X, bias, out, M, N, K, NT, TT);
        break;
      default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
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
