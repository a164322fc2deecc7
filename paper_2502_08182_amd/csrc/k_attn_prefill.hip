// Prefill attention: causal attention of a sequence's new tokens over its cached and
// new keys, on the matrix cores (prefill is the computation-intensive phase, paper
// Sec. 2.1).  One 256-thread workgroup handles kPrefillQTile = 128 query rows of one
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

hipError_t launch_attn_prefill(int dtype, const void* qkv16, const void* kv, const StepIndex& ix, void* out16,
                               int n_qtiles, int Hq, int Hkv, int d, hipStream_t st, int packed) {
  if (n_qtiles <= 0) return hipSuccess;
  if (packed && (Hq * d) % 32) return hipErrorInvalidValue;
  dim3 grid(n_qtiles, Hq), block(256);
#define SN_PREFILL(TT, DD)                                                                                    \
  SN_LAUNCH((attn_prefill_kernel<TT, DD>), grid, block, 0, st, (const uint16_t*)qkv16,               \
                     (const uint16_t*)kv, ix.len_before, ix.n_new, ix.tok_start, ix.kv_off, ix.cap, ix.tile_seq, \
                     ix.tile_q0, (uint16_t*)out16, Hq, Hkv, packed)
  if (dtype == 0 && d == 64) SN_PREFILL(F16, 64);
  else if (dtype == 0 && d == 128) SN_PREFILL(F16, 128);
  else if (dtype == 1 && d == 64) SN_PREFILL(BF16, 64);
  else if (dtype == 1 && d == 128) SN_PREFILL(BF16, 128);
  else return hipErrorInvalidValue;
#undef SN_PREFILL
  return hipGetLastError();
}

}  // namespace sn
