// Prefill attention: causal attention of a sequence's new tokens over its cached and
// new keys, on the matrix cores (prefill is the computation-intensive phase, paper
// Sec. 2.1).  Two kernels: attn_prefill128_kernel (head dimension 128, further down; every
// full-size workload) and attn_prefill_kernel (any head dimension the library takes; in use for 64),
// described here.  One 256-thread workgroup handles kPrefillQTile = 128 query rows of one
// (sequence, query head); each wavefront owns 32 of them as two 16-query MFMA column tiles, so
// every K and V fragment read from LDS feeds two products.  Keys are consumed 32 at a time,
// staged through a pair of LDS tiles (K row-major, V transposed) shared by the four wavefronts:
//
//   S^T = K Q^T   A operand = 16 key rows x 32 of d (read from the LDS K tile),
//                 B operand = Q^T (this wavefront's 16 queries), result D[key][query].
//                 The 16 rows of the two key sub-tiles are chosen as keys
//                 8*(r/4) + 4*t + r%4 so that a lane ends up holding the scores of
//                 8 *consecutive* keys (8*(lane/16) .. +8) for query lane%16 --
//                 exactly the B-operand layout the next product needs.
//   O^T = V^T P^T A operand = V^T (16 of d x 32 keys) read from an LDS tile that was
//                 transposed while being staged, B operand = P^T from registers,
//                 result D[d][query]: the query index stays on lane%16, so the online
//                 softmax rescale is lane-local.
#include "kernels.h"
#include "common.h"

namespace sn {

constexpr float kMasked = -1.0e30f;

template <class T, int D>
__global__ __launch_bounds__(256) void attn_prefill_kernel(
    const uint16_t* __restrict__ qkv, const uint16_t* __restrict__ kv, const int32_t* __restrict__ len_before,
    const int32_t* __restrict__ n_new, const int32_t* __restrict__ tok_start, const int32_t* __restrict__ kv_off,
    const int32_t* __restrict__ cap, const int32_t* __restrict__ tile_seq, const int32_t* __restrict__ tile_q0,
    uint16_t* __restrict__ out, int Hq, int Hkv, int packed) {
  constexpr int KT = 32;              // keys per step
  constexpr int LD = 40;              // LDS row stride (elements) of the transposed V tile: 80 B, 16 B aligned
  constexpr int LDK = D + 8;          // LDS row stride (elements) of the K tile: rows 16 B apart modulo 256 B
  constexpr int DK = D / 32;          // k-steps over the head dimension
  constexpr int DT = D / 16;          // 16-wide output tiles over the head dimension
  constexpr int RING = 2;             // key tiles in LDS: the one being computed and the next one, written at the end of the step
  constexpr int QW = kPrefillQTile / 64;  // 16-query tiles per wavefront
  constexpr int KCH = KT * (D / 8) / 256;   // 16-byte pieces of the K tile per thread (2 at d = 128, 1 at d = 64)
  static_assert(KCH >= 1 && KT * (D / 8) % 256 == 0, "K tile must split evenly over the workgroup");
  __shared__ __attribute__((aligned(16))) uint16_t ks[RING][KT * LDK];
  __shared__ __attribute__((aligned(16))) uint16_t vt[RING][D * LD];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  // tiles are listed per sequence with the first query rising, i.e. with the causal work rising: take them
  // from the back so that the longest workgroups start first and the short ones fill the end of the launch
  const int tile = gridDim.x - 1 - blockIdx.x;
  const int b = tile_seq[tile];
  const int q0 = tile_q0[tile];
  const int hq = blockIdx.y;
  const int hk = hq / (Hq / Hkv);
  const int nn = n_new[b];
  const int lb = len_before[b];
  const int total = lb + nn;                             // keys that exist after the append
  const int kend = lb + min(nn, q0 + kPrefillQTile);     // keys any query of this tile may see

  const int qkv_ld = (Hq + 2 * Hkv) * D;
  const int qw0 = q0 + wave * 16 * QW;                   // first query (new-token index) of this wavefront
  int qi[QW], qpos[QW];                                  // this lane's query in each of its column tiles
  bool qok[QW];
  u16x8 qf[QW][DK];
#pragma unroll
  for (int j = 0; j < QW; ++j) {
    qi[j] = qw0 + j * 16 + r;
    qok[j] = qi[j] < nn;
    qpos[j] = lb + qi[j];
#pragma unroll
    for (int kk = 0; kk < DK; ++kk) {
      qf[j][kk] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
      if (qok[j])
        qf[j][kk] = *reinterpret_cast<const u16x8*>(qkv + (size_t)(tok_start[b] + qi[j]) * qkv_ld + (size_t)hq * D +
                                                    kk * 32 + g * 8);
    }
  }

  const int cp = cap[b];
  const uint16_t* Kb = kv + (size_t)kv_off[b] * 2 * Hkv * D + (size_t)(hk * 2) * cp * D;
  const uint16_t* Vb = Kb + (size_t)cp * D;
  const float scale2 = rsqrtf((float)D) * 1.4426950408889634f;   // log2(e) / sqrt(d)
  const int qlo = lb + qw0;                              // position of this wavefront's first query

  float m[QW], l[QW];
  f32x4 o[QW][DT];
#pragma unroll
  for (int j = 0; j < QW; ++j) {
    m[j] = kMasked;
    l[j] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[j][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // A key tile travels global -> registers -> LDS.  Its loads are issued two steps before it is
  // computed and it is written to LDS at the end of the step before (two register sets, two LDS
  // tiles, one barrier per step: the tile overwritten was last read one barrier ago), so a load
  // has two steps of arithmetic to hide behind.  K goes
  // to LDS row-major, shared by the four wavefronts; V as (key pair, 8 d-values) items that are
  // transposed on the way in.
  constexpr int ITEMS = (KT / 2) * (D / 8);              // <= 256: at most one V item per thread
  static_assert(ITEMS <= 256, "one V item per thread");
  const bool vitem = (int)threadIdx.x < ITEMS;
  const int vkey = 2 * (threadIdx.x & 15), vdc = threadIdx.x >> 4;
  const int kkey = (threadIdx.x * KCH) / (D / 8), kch = (threadIdx.x * KCH) % (D / 8);   // K row and first piece
  struct Stage {
    u16x8 k[KCH], va, vb;
  };
  auto gload = [&](int j0, Stage& R) {
    R.va = R.vb = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
    if (vitem && j0 + vkey < total) R.va = *reinterpret_cast<const u16x8*>(Vb + (size_t)(j0 + vkey) * D + vdc * 8);
    if (vitem && j0 + vkey + 1 < total) R.vb = *reinterpret_cast<const u16x8*>(Vb + (size_t)(j0 + vkey + 1) * D + vdc * 8);
    const int key = min(j0 + kkey, total - 1);           // inside the cached rows; masked later
#pragma unroll
    for (int c = 0; c < KCH; ++c) R.k[c] = *reinterpret_cast<const u16x8*>(Kb + (size_t)key * D + (kch + c) * 8);
  };
  auto lstore = [&](int buf, const Stage& R) {
#pragma unroll
    for (int c = 0; c < KCH; ++c) *reinterpret_cast<u16x8*>(&ks[buf][kkey * LDK + (kch + c) * 8]) = R.k[c];
    if (vitem) {
      // vt[dcol][key], eight 4-byte writes {v[key][e], v[key+1][e]}
      const u16x8 ra = rot_pairs(R.va, g), rb = rot_pairs(R.vb, g);
#pragma unroll
      for (int e0 = 0; e0 < 8; ++e0) {
        const int e = (e0 + 2 * g) & 7;                  // 16-lane groups write different rows: fewer bank conflicts
        *reinterpret_cast<uint32_t*>(&vt[buf][(vdc * 8 + e) * LD + vkey]) = (uint32_t)ra[e0] | ((uint32_t)rb[e0] << 16);
      }
    }
  };
  auto compute = [&](int buf, int j0) {
    if (j0 > qlo + 16 * QW - 1) return;                  // every key of this tile lies after all of this wavefront's queries
    // ---- scores of 32 keys for this wavefront's 16 * QW queries ----
    f32x4 st[QW][2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int j = 0; j < QW; ++j) st[j][t] = f32x4{0.f, 0.f, 0.f, 0.f};
      const uint16_t* kp = &ks[buf][(8 * (r >> 2) + 4 * t + (r & 3)) * LDK + g * 8];
#pragma unroll
      for (int kk = 0; kk < DK; ++kk) {
        const u16x8 kfrag = *reinterpret_cast<const u16x8*>(kp + kk * 32);
#pragma unroll
        for (int j = 0; j < QW; ++j) st[j][t] = mma16x16x32<T>(kfrag, qf[j][kk], st[j][t]);
      }
    }
    u16x8 pb[QW];
#pragma unroll
    for (int j = 0; j < QW; ++j) {
      // lane now holds scores of keys j0 + 8g + e (e = 4t + i) for query lane%16 of column tile j.  The
      // softmax runs in the base-2 domain (scores times log2 e / sqrt d, v_exp_f32 is 2^x).  Away from
      // the diagonal and the ragged end of the sequence nothing needs masking (decided per wavefront).
      float sc[8];
      float mx = kMasked;
      if (qw0 + j * 16 + 15 < nn && j0 + KT - 1 <= qlo + j * 16) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          sc[e] = st[j][e >> 2][e & 3] * scale2;
          mx = fmaxf(mx, sc[e]);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int key = j0 + 8 * g + e;
          const bool ok = qok[j] && key <= qpos[j];
          sc[e] = ok ? st[j][e >> 2][e & 3] * scale2 : kMasked;
          mx = fmaxf(mx, sc[e]);
        }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // the running maximum rarely moves after the first tiles: rescale only when it does for some
      // query of the wavefront (multiplying by 2^0 would change nothing)
      if (__any(mx > m[j])) {
        const float mn = fmaxf(m[j], mx);
        const float corr = __builtin_amdgcn_exp2f(m[j] - mn);
        l[j] *= corr;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int i = 0; i < 4; ++i) o[j][dt][i] *= corr;
        m[j] = mn;
      }
      float rs = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // a masked score is -1e30: 2^(-1e30 - m) is 0 once the row has seen a real key, which its
        // first tile always holds (key 0); rows of queries past the end are never stored
        const float p = __builtin_amdgcn_exp2f(sc[e] - m[j]);
        rs += p;
        pb[j][e] = from_f32<T>(p);
      }
      l[j] += rs;                                        // per-lane partial; lanes of a query are summed at the end
    }
    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const u16x8 vf = *reinterpret_cast<const u16x8*>(&vt[buf][(dt * 16 + r) * LD + g * 8]);
#pragma unroll
      for (int j = 0; j < QW; ++j) o[j][dt] = mma16x16x32<T>(vf, pb[j], o[j][dt]);
    }
  };

  const int nsteps = (kend + KT - 1) / KT;
  Stage RA, RB;
  if (nsteps > 0) {
    gload(0, RA);
    if (nsteps > 1) gload(KT, RB);
    lstore(0, RA);
  }
  __syncthreads();
  // step t: tile t is in LDS slot t % RING, tile t + 1 is arriving in `next`; tile t + 2 is requested into `far`
  // (which held tile t, already in LDS), tile t is computed, tile t + 1 goes to its LDS slot.
  auto step = [&](int t, Stage& far, const Stage& next) {
    if (t + 2 < nsteps) gload((t + 2) * KT, far);
    compute(t % RING, t * KT);
    if (t + 1 < nsteps) lstore((t + 1) % RING, next);
    __syncthreads();
  };
  for (int t = 0; t < nsteps; t += 2) {
    step(t, RA, RB);
    if (t + 1 < nsteps) step(t + 1, RB, RA);
  }

#pragma unroll
  for (int j = 0; j < QW; ++j) {
    float lj = l[j];
    lj += __shfl_xor(lj, 16, 64);
    lj += __shfl_xor(lj, 32, 64);
    if (qok[j]) {
      const float inv = 1.0f / lj;
      const int tok = tok_start[b] + qi[j];
      uint16_t* op = out + (size_t)tok * Hq * D + (size_t)hq * D + g * 4;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        u16x4 w;
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = from_f32<T>(o[j][dt][i] * inv);
        if (packed)       // row-tile packed (feeds the output projection): 16 tokens x 16 bytes are contiguous
          *reinterpret_cast<u16x4*>(out + packed_off(tok, hq * D + dt * 16 + g * 4, (Hq * D) >> 5)) = w;
        else
          *reinterpret_cast<u16x4*>(op + dt * 16) = w;
      }
    }
  }
}

// ---------------------------------------------------------------------------------
// Head dimension 128 (every full-size workload): 32 x 32 x 16 matrix-core tiles
// ---------------------------------------------------------------------------------
// Same split of the work (128 query rows of one (sequence, head) per workgroup, 32 per wavefront), but the
// two products run on 32 x 32 x 16 tiles and a step covers 64 keys: each operand element read from LDS feeds
// twice the arithmetic of a 16 x 16 x 32 tile, and everything that happens once per step and query (maximum
// across lanes, the moved-maximum test, the barrier, address arithmetic) is paid for half as often.
//
//   S^T = K Q^T   A operand: 32 keys x 16 of d from the LDS K tile (row-major, rows 272 bytes apart, so the 16
//                 lanes of a 128-bit read hit 16 different bank groups), B operand: Q^T from registers.
//                 Lane l receives, for query l % 32, the keys 8*(v/4) + 4*(l/32) + v%4, v = 0..15 of each 32-key block.
//   O^T = V^T P^T the k index of a product may be numbered in any order as long as both operands agree: k slot
//                 (l/32, e) of product c2 (16 keys of block c) is key 16*c2 + 8*(e/4) + 4*(l/32) + e%4, which makes
//                 the B operand exactly the eight score registers v = 8*c2 .. 8*c2 + 7 of the lane, no movement.
//                 The A operand, V^T, comes from an LDS tile [d][key slot] written in that same slot order, so a
//                 lane's eight values are one 16-byte unit; units are xor-swizzled with the row so that both the
//                 transposing writes (8 bytes: four keys of one d) and the 128-bit reads spread over the banks.
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <class T> __device__ __forceinline__ f32x16 mma32x32x16(u16x8 a, u16x8 b, f32x16 c);
template <> __device__ __forceinline__ f32x16 mma32x32x16<F16>(u16x8 a, u16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x16 mma32x32x16<BF16>(u16x8 a, u16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// 16-byte unit of V^T row r that holds key-slot unit u (0..7)
__device__ __forceinline__ int vt_unit(int r, int u) { return u ^ (((r >> 1) ^ (r >> 4)) & 7); }

template <class T>
__global__ __launch_bounds__(256, 2) void attn_prefill128_kernel(
    const uint16_t* __restrict__ qkv, const uint16_t* __restrict__ kv, const int32_t* __restrict__ len_before,
    const int32_t* __restrict__ n_new, const int32_t* __restrict__ tok_start, const int32_t* __restrict__ kv_off,
    const int32_t* __restrict__ cap, const int32_t* __restrict__ tile_seq, const int32_t* __restrict__ tile_q0,
    uint16_t* __restrict__ out, int Hq, int Hkv, int packed, int n_qtiles) {
  constexpr int D = 128;
  constexpr int KT = 64;              // keys per step
  constexpr int RSK = D + 8;          // K tile row stride (elements)
  constexpr int QW = 32;              // queries per wavefront
  static_assert(kPrefillQTile == 4 * QW, "four wavefronts of 32 queries");
  __shared__ __attribute__((aligned(16))) uint16_t ks[2][KT * RSK];
  __shared__ __attribute__((aligned(16))) uint16_t vt[2][D * KT];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int qc = lane & 31, half = lane >> 5;
  // Workgroup id -> (query tile, head).  Work items are numbered KV head by KV head, inside a KV head tile by tile from
  // the back of the list (tiles are listed per sequence with the first query rising: the longest of a sequence come
  // first, the short ones of the first sequence fill the end of the launch), inside a tile over the query heads that
  // share the KV head.  Hardware deals consecutive workgroup ids round-robin to the 8 XCDs; XCD x takes the x-th
  // eighth of that numbering in order, so the ~64 workgroups it runs at once are neighbouring tiles and heads of one
  // (sequence, KV head) and find its K and V in that XCD's L2 (numbered head-major, tile-fastest, the workgroups in
  // flight covered every sequence at once and four K / V reads out of five missed the L2).
  const int G = Hq / Hkv;
  const int n_items = n_qtiles * Hq, chunk = (n_items + 7) >> 3;
  const int item = (blockIdx.x & 7) * chunk + (blockIdx.x >> 3);
  if (item >= n_items) return;
  const int hk = item / (n_qtiles * G), rem = item - hk * (n_qtiles * G);
  const int tile = n_qtiles - 1 - rem / G;
  const int hq = hk * G + rem % G;
  const int b = tile_seq[tile];
  const int q0 = tile_q0[tile];
  const int nn = n_new[b];
  const int lb = len_before[b];
  const int total = lb + nn;
  const int kend = lb + min(nn, q0 + kPrefillQTile);

  const int qkv_ld = (Hq + 2 * Hkv) * D;
  const int qw0 = q0 + wave * QW;                        // first query (new-token index) of this wavefront
  const int qi = qw0 + qc;
  const bool qok = qi < nn;
  const int qpos = lb + qi;
  const int qlo = lb + qw0;
  u16x8 qf[D / 16];                                      // B operand: query qc, d = 16*kk + 8*half .. +8
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) {
    qf[kk] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
    if (qok)
      qf[kk] = *reinterpret_cast<const u16x8*>(qkv + (size_t)(tok_start[b] + qi) * qkv_ld + (size_t)hq * D + kk * 16 + half * 8);
  }

  const int cp = cap[b];
  const uint16_t* Kb = kv + (size_t)kv_off[b] * 2 * Hkv * D + (size_t)(hk * 2) * cp * D;
  const uint16_t* Vb = Kb + (size_t)cp * D;
  const float scale2 = rsqrtf((float)D) * 1.4426950408889634f;   // log2(e) / sqrt(d)

  float m = kMasked, l = 0.f;
  f32x16 o[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;

  // Staging, one step ahead: global -> registers while the previous tile is computed, registers -> LDS at the end of
  // that step.  K: thread t moves the 16-byte piece t % 16 of rows t / 16 + 16 i.  V: thread t moves d-chunk t % 16 of
  // the four consecutive keys 4 * (t / 16) .. + 3 (whole 256-byte rows per 16 lanes), transposes the 4 x 8 block in
  // registers and writes, for each of its 8 values of d, the four keys as one 8-byte piece of that V^T row.
  const int kch = threadIdx.x & 15, krow = threadIdx.x >> 4;
  const int vdc = threadIdx.x & 15, vkg = threadIdx.x >> 4;
  // key group -> (32-key block c, product c2, 8-key half j, lane half): 4 * kg = 32 c + 16 c2 + 8 j + 4 hf
  const int vunit = ((vkg >> 3) << 2) | (((vkg >> 2) & 1) << 1) | (vkg & 1);
  const int vj = (vkg >> 1) & 1;
  struct Stage {
    u16x8 k[4], v[4];
  };
  auto gload = [&](int j0, Stage& R) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int key = min(j0 + krow + 16 * i, total - 1);          // inside the cached rows; masked later
      R.k[i] = *reinterpret_cast<const u16x8*>(Kb + (size_t)key * D + kch * 8);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int key = min(j0 + 4 * vkg + i, total - 1);
      R.v[i] = *reinterpret_cast<const u16x8*>(Vb + (size_t)key * D + vdc * 8);
    }
  };
  auto lstore = [&](int buf, int j0, const Stage& R) {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u16x8*>(&ks[buf][(krow + 16 * i) * RSK + kch * 8]) = R.k[i];
    u32x4 w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = __builtin_bit_cast(u32x4, R.v[i]);
    if (j0 + KT > total) {                               // rows past the end must not carry NaN into 0 * v
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (j0 + 4 * vkg + i >= total) w[i] = u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int mm = 0; mm < 4; ++mm) {
      // dword mm of each key holds d = 2 mm (low half) and 2 mm + 1 (high half)
      u32x2 lo, hi;
      lo[0] = __builtin_amdgcn_perm(w[1][mm], w[0][mm], 0x05040100u);
      lo[1] = __builtin_amdgcn_perm(w[3][mm], w[2][mm], 0x05040100u);
      hi[0] = __builtin_amdgcn_perm(w[1][mm], w[0][mm], 0x07060302u);
      hi[1] = __builtin_amdgcn_perm(w[3][mm], w[2][mm], 0x07060302u);
      const int r0 = vdc * 8 + 2 * mm, r1 = r0 + 1;
      *reinterpret_cast<u32x2*>(&vt[buf][r0 * KT + vt_unit(r0, vunit) * 8 + vj * 4]) = lo;
      *reinterpret_cast<u32x2*>(&vt[buf][r1 * KT + vt_unit(r1, vunit) * 8 + vj * 4]) = hi;
    }
  };
  auto compute = [&](int buf, int j0) {
    if (j0 > qlo + QW - 1) return;                       // every key of this tile lies after all of this wavefront's queries
    // ---- scores of 64 keys (two 32-key blocks) for this wavefront's 32 queries ----
    f32x16 st[2];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < 16; ++i) st[c][i] = 0.f;
    const uint16_t* kp = &ks[buf][qc * RSK + half * 8];
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const u16x8 kf = *reinterpret_cast<const u16x8*>(kp + c * 32 * RSK + kk * 16);
        st[c] = mma32x32x16<T>(kf, qf[kk], st[c]);
      }
    }
    // lane holds, for query qc, the raw scores of keys j0 + 32 c + 8 (i / 4) + 4 half + i % 4.  Away from the
    // diagonal and the ragged end nothing needs masking (decided per wavefront).
    if (!(qw0 + QW - 1 < nn && j0 + KT - 1 <= qlo)) {
      // key offset inside the tile (without the lane half) must be <= lim.  Rows of queries past the end are never
      // stored; their q is zero, and left unmasked they stay finite (all scores 0) instead of 2^(rounding of -1e30)
      const int lim = qok ? qpos - j0 - 4 * half : KT;
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (32 * c + 8 * (i >> 2) + (i & 3) > lim) st[c][i] = kMasked;
    }
    float mx = kMasked;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, st[c][i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    mx *= scale2;                                        // the softmax runs in the base-2 domain
    // the running maximum rarely moves after the first tiles: rescale only when it does for some query of the wavefront
    if (__any(mx > m)) {
      const float mn = fmaxf(m, mx);
      const float corr = __builtin_amdgcn_exp2f(m - mn);
      l *= corr;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= corr;
      m = mn;
    }
    // a masked score is -1e30: 2^(-1e30 * scale - m) is 0 once the row has seen a real key, which its first tile
    // always holds (key 0)
    u16x8 pb[2][2];
    float rs = 0.f;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(st[c][i], scale2, -m));
        rs += p;
        pb[c][i >> 3][i & 7] = from_f32<T>(p);
      }
    l += rs;                                             // per-lane partial; the two lanes of a query are summed at the end
    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
      const int r = db * 32 + qc;
      const uint16_t* vp = &vt[buf][r * KT];
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2) {
          const u16x8 vf = *reinterpret_cast<const u16x8*>(vp + vt_unit(r, c * 4 + c2 * 2 + half) * 8);
          o[db] = mma32x32x16<T>(vf, pb[c][c2], o[db]);
        }
    }
  };

  // kend >= 1, so there is a first tile.  Its store to LDS waits for every load issued so far, the query fragments
  // included, on the only path into the loop: the waits the compiler places inside the loop then count the one tile
  // in flight and nothing older (a path around that wait made it wait for all loads at the top of every step).
  const int nsteps = (kend + KT - 1) / KT;
  Stage R;
  gload(0, R);
  lstore(0, 0, R);
  if (nsteps > 1) gload(KT, R);
  __syncthreads();
  for (int t = 0; t < nsteps; ++t) {
    compute(t & 1, t * KT);
    if (t + 1 < nsteps) lstore((t + 1) & 1, (t + 1) * KT, R);   // that buffer was last read one barrier ago
    if (t + 2 < nsteps) gload((t + 2) * KT, R);
    __syncthreads();
  }

  l += __shfl_xor(l, 32, 64);
  if (qok) {
    const float inv = 1.0f / l;
    const int tok = tok_start[b] + qi;
    uint16_t* op = out + (size_t)tok * Hq * D + (size_t)hq * D;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int dcol = db * 32 + i4 * 8 + half * 4;
        u16x4 w;
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = from_f32<T>(o[db][i4 * 4 + i] * inv);
        if (packed)       // row-tile packed (feeds the output projection)
          *reinterpret_cast<u16x4*>(out + packed_off(tok, hq * D + dcol, (Hq * D) >> 5)) = w;
        else
          *reinterpret_cast<u16x4*>(op + dcol) = w;
      }
  }
}


hipError_t launch_attn_prefill(int dtype, const void* qkv16, const void* kv, const StepIndex& ix, void* out16,
                               int n_qtiles, int Hq, int Hkv, int d, hipStream_t st, int packed) {
  if (n_qtiles <= 0) return hipSuccess;
  if (packed && (Hq * d) % 32) return hipErrorInvalidValue;
  dim3 grid(n_qtiles, Hq), block(256);
#define SN_PREFILL(TT, DD)                                                                                    \
  SN_LAUNCH((attn_prefill_kernel<TT, DD>), grid, block, 0, st, (const uint16_t*)qkv16,               \
                     (const uint16_t*)kv, ix.len_before, ix.n_new, ix.tok_start, ix.kv_off, ix.cap, ix.tile_seq, \
                     ix.tile_q0, (uint16_t*)out16, Hq, Hkv, packed)
  dim3 grid128(8 * ((n_qtiles * Hq + 7) / 8));
#define SN_PREFILL128(TT)                                                                                    \
  SN_LAUNCH((attn_prefill128_kernel<TT>), grid128, block, 0, st, (const uint16_t*)qkv16,               \
                     (const uint16_t*)kv, ix.len_before, ix.n_new, ix.tok_start, ix.kv_off, ix.cap, ix.tile_seq, \
                     ix.tile_q0, (uint16_t*)out16, Hq, Hkv, packed, n_qtiles)
  if (dtype == 0 && d == 64) SN_PREFILL(F16, 64);
  else if (dtype == 0 && d == 128) SN_PREFILL128(F16);
  else if (dtype == 1 && d == 64) SN_PREFILL(BF16, 64);
  else if (dtype == 1 && d == 128) SN_PREFILL128(BF16);
  else return hipErrorInvalidValue;
#undef SN_PREFILL
#undef SN_PREFILL128
  return hipGetLastError();
}

}  // namespace sn
