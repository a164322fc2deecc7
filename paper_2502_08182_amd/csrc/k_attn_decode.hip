// Decode attention: one query per sequence against its cached keys and values.
//
// Memory-bound (paper Sec. 2.1, decoding): every cached K and V element is read once.
// The KV slice keeps, for each (sequence, KV head), K rows [cap][d] and then V rows
// [cap][d], so a workgroup assigned to one (sequence, KV head, key range) streams two
// contiguous regions.  Lanes are laid along the head dimension: d/8 lanes share one key
// row (16 bytes each), so one wavefront load covers 64/(d/8) consecutive keys = 1 KiB.
// The dot product is finished with xor-shuffles inside those d/8 lanes; every
// (wavefront, key slot) keeps its own running softmax (max, sum, weighted V), merged
// at the end by shuffles, then across the wavefronts through LDS, then across key
// ranges by a second small kernel.  All merges run in a fixed order.
//
// Three kernels: attn_decode_gqa128_kernel (head dimension 128, 1 to 8 query heads per KV
// head: matrix cores, whole-line loads -- what every configuration measured here runs),
// attn_decode_gqa_kernel (head dimension 64, 4 or 8 query heads per KV head: matrix cores,
// V^T staged through LDS) and attn_decode_kernel (head dimension 64, 1 or 2 query heads per
// KV head: the vector kernel described above).
#include "kernels.h"
#include "common.h"

namespace sn {

constexpr float kNegBig = -1.0e30f;

// Fused append (template flag FA): the decode step's own q, k and v rows are still
// un-rotated in the QKV projection's output.  The workgroup rotates q and k (RoPE,
// pairs (i, i + d/2), fp32 angles), rounds them to the 16-bit storage type and parks
// them in LDS: rows 0..G-1 = the group's query heads, row G = k, row G+1 = v.  The key
// range that contains the new position stores k and v into the KV slice (and its host
// mirror, when the layer's KV lives in host memory) and takes that key from LDS instead
// of from the cache, so no workgroup ever loads the row that is being written.
//
// When the QKV projection ran split over K (few output features: the only way to give every
// compute unit a workgroup), its output arrives as fp32 partial planes instead: qpart
// [nsplit][rows][(Hq + 2 Hkv) d], bias already in plane 0.  The planes are summed here in
// ascending order and the sum is rounded to the 16-bit type first -- exactly the value the
// unsplit projection would have stored -- so everything after this point is unchanged.
struct QkvPlanes {
  const float* part;     // null: read the 16-bit row
  int nsplit;
  int rows;              // rows of one plane
};
template <class T, int D, int G>
__device__ __forceinline__ void stage_new_token(uint16_t (*stage)[D], const uint16_t* __restrict__ qkv_row,
                                                const QkvPlanes qp, int seq, int hk, int Hq, int Hkv, int pos,
                                                const float* __restrict__ inv_freq, int rope) {
  constexpr int half = D / 2;
  const int ld = (Hq + 2 * Hkv) * D;
  for (int t = threadIdx.x; t < (G + 2) * half; t += blockDim.x) {
    const int hs = t / half, i = t % half;
    const int head = hs < G ? hk * G + hs : hs == G ? Hq + hk : Hq + Hkv + hk;
    float a, b;
    if (qp.part) {
      const float* src = qp.part + (size_t)seq * ld + (size_t)head * D;
      const size_t plane = (size_t)qp.rows * ld;
      // all planes requested at once (absent ones read as zero), then added in ascending order
      float va[kMaxSplits], vb[kMaxSplits];
#pragma unroll
      for (int sp = 0; sp < kMaxSplits; ++sp) {
        const bool on = sp < qp.nsplit;
        va[sp] = on ? src[sp * plane + i] : 0.f;
        vb[sp] = on ? src[sp * plane + i + half] : 0.f;
      }
      float sa = va[0], sb = vb[0];
#pragma unroll
      for (int sp = 1; sp < kMaxSplits; ++sp) {
        sa += va[sp];
        sb += vb[sp];
      }
      a = to_f32<T>(from_f32<T>(sa));
      b = to_f32<T>(from_f32<T>(sb));
    } else {
      const uint16_t* src = qkv_row + (size_t)head * D;
      a = to_f32<T>(src[i]);
      b = to_f32<T>(src[i + half]);
    }
    if (rope && hs <= G) {
      float sn_, cs_;
      sincosf((float)pos * inv_freq[i], &sn_, &cs_);
      const float ra = a * cs_ - b * sn_;
      const float rb = a * sn_ + b * cs_;
      a = ra;
      b = rb;
    }
    stage[hs][i] = from_f32<T>(a);
    stage[hs][i + half] = from_f32<T>(b);
  }
}

// k and v of the new position: LDS rows G and G+1 -> KV slice row `pos` (16-byte stores).
template <int D, int G>
__device__ __forceinline__ void store_new_token(const uint16_t (*stage)[D], uint16_t* __restrict__ kvw,
                                                uint16_t* __restrict__ mirror, size_t k_row_off, size_t v_row_off) {
  constexpr int LPK = D / 8;
  if (threadIdx.x < 2 * LPK) {
    const int is_v = threadIdx.x / LPK, cc = threadIdx.x % LPK;
    const u16x8 val = *reinterpret_cast<const u16x8*>(&stage[G + is_v][cc * 8]);
    const size_t off = (is_v ? v_row_off : k_row_off) + cc * 8;
    *reinterpret_cast<u16x8*>(kvw + off) = val;
    if (mirror) *reinterpret_cast<u16x8*>(mirror + off) = val;
  }
}

__device__ __forceinline__ void merge_into(float& m, float& l, float (&a)[8], float m2, float l2,
                                           const float (&a2)[8]) {
  const float mn = fmaxf(m, m2);
  const float c1 = __expf(m - mn), c2 = __expf(m2 - mn);
  l = l * c1 + l2 * c2;
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] = a[e] * c1 + a2[e] * c2;
  m = mn;
}

// NW wavefronts per workgroup, UK key groups (one wavefront load each for K and V) in
// flight per wavefront.  Measured on MI355X: 16 x 2 is best for multi-head attention at
// small batch (8 x 32 heads x 530 keys: 14.9 us vs 16.8 us for 8 x 4); with 8 query heads
// per KV head the per-lane state needs the registers of an 8-wavefront workgroup.
template <class T, int D, int G, int NW, int UK, bool FA>
__global__ __launch_bounds__(NW * 64) void attn_decode_kernel(
    const uint16_t* __restrict__ qkv, const uint16_t* __restrict__ kv, const int32_t* __restrict__ len_before,
    const int32_t* __restrict__ kv_off, const int32_t* __restrict__ cap, uint16_t* __restrict__ out,
    float* __restrict__ part, int Hq, int Hkv, int S, int packed, uint16_t* __restrict__ kvw,
    uint16_t* __restrict__ mirror, const float* __restrict__ inv_freq, int rope, QkvPlanes qp) {
  constexpr int LPK = D / 8;          // lanes per key row
  constexpr int KPW = 64 / LPK;       // keys per wavefront load
  __shared__ float lds[NW][G][LPK][10];
  __shared__ __attribute__((aligned(16))) uint16_t stage[FA ? G + 2 : 1][D];

  const int b = blockIdx.x / Hkv;
  const int hk = blockIdx.x % Hkv;
  const int split = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int slot = lane / LPK, c = lane % LPK;

  const int len = len_before[b] + 1;
  const int chunk = (len + S - 1) / S;
  const int j0 = split * chunk;
  const int j1 = min(len, j0 + chunk);

  const int qkv_ld = (Hq + 2 * Hkv) * D;
  const float scale = rsqrtf((float)D);
  const int cp = cap[b];
  const size_t k_base = (size_t)kv_off[b] * 2 * Hkv * D + (size_t)(hk * 2) * cp * D;
  const int pos = len - 1;            // position of this step's token
  u16x8 knew = {0, 0, 0, 0, 0, 0, 0, 0}, vnew = {0, 0, 0, 0, 0, 0, 0, 0};
  if (FA) {
    stage_new_token<T, D, G>(stage, qkv + (size_t)b * qkv_ld, qp, b, hk, Hq, Hkv, pos, inv_freq, rope);
    __syncthreads();
    if (pos >= j0 && pos < j1)
      store_new_token<D, G>(stage, kvw, mirror, k_base + (size_t)pos * D, k_base + ((size_t)cp + pos) * D);
    knew = *reinterpret_cast<const u16x8*>(&stage[G][c * 8]);
    vnew = *reinterpret_cast<const u16x8*>(&stage[G + 1][c * 8]);
  }
  float q[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const u16x8 v = FA ? *reinterpret_cast<const u16x8*>(&stage[g][c * 8])
                       : *reinterpret_cast<const u16x8*>(qkv + (size_t)b * qkv_ld + (size_t)(hk * G + g) * D + c * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) q[g][e] = to_f32<T>(v[e]) * scale;
  }

  const uint16_t* Kb = kv + k_base + c * 8;
  const uint16_t* Vb = Kb + (size_t)cp * D;
  // last cached row a load may touch: with the fused append the new row is never loaded
  const int jlast = FA ? max(min(j1 - 1, pos - 1), 0) : j1 - 1;

  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = kNegBig;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
  }

  // wavefront `wave` takes key groups wave, wave+NW, ...; UK groups per trip are loaded
  // before any is used so that 2*UK KiB per wavefront are in flight
  for (int jb = j0 + wave * KPW; jb < j1; jb += NW * KPW * UK) {
    u16x8 kr[UK], vr[UK];
    bool ok[UK];
#pragma unroll
    for (int u = 0; u < UK; ++u) {
      const int j = jb + u * NW * KPW + slot;
      ok[u] = j < j1;
      const int jc = min(j, jlast);                    // clamped: loads stay inside the cached rows
      kr[u] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(Kb + (size_t)jc * D));
      vr[u] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(Vb + (size_t)jc * D));
      if (FA && j == pos) {
        kr[u] = knew;
        vr[u] = vnew;
      }
    }
#pragma unroll
    for (int u = 0; u < UK; ++u) {
      float kf[8], vf[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        kf[e] = to_f32<T>(kr[u][e]);
        vf[e] = to_f32<T>(vr[u][e]);
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s += q[g][e] * kf[e];
#pragma unroll
        for (int o = LPK / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        if (ok[u]) {
          const float mn = fmaxf(m[g], s);
          const float corr = __expf(m[g] - mn);
          const float p = __expf(s - mn);
          l[g] = l[g] * corr + p;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[g][e] = acc[g][e] * corr + p * vf[e];
          m[g] = mn;
        }
      }
    }
  }

  // merge the key slots of this wavefront (lanes that hold the same d-chunk)
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int o = LPK; o < 64; o <<= 1) {
      const float m2 = __shfl_xor(m[g], o, 64);
      const float l2 = __shfl_xor(l[g], o, 64);
      float a2[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) a2[e] = __shfl_xor(acc[g][e], o, 64);
      merge_into(m[g], l[g], acc[g], m2, l2, a2);
    }
    if (slot == 0) {
      lds[wave][g][c][0] = m[g];
      lds[wave][g][c][1] = l[g];
#pragma unroll
      for (int e = 0; e < 8; ++e) lds[wave][g][c][2 + e] = acc[g][e];
    }
  }
  __syncthreads();

  // merge the wavefronts in order: thread (g, c)
  if (threadIdx.x < G * LPK) {
    const int g = threadIdx.x / LPK, cc = threadIdx.x % LPK;
    float mm = lds[0][g][cc][0], ll = lds[0][g][cc][1], aa[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) aa[e] = lds[0][g][cc][2 + e];
    for (int w = 1; w < NW; ++w) {
      float a2[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) a2[e] = lds[w][g][cc][2 + e];
      merge_into(mm, ll, aa, lds[w][g][cc][0], lds[w][g][cc][1], a2);
    }
    const int hq = hk * G + g;
    if (S == 1) {
      const float inv = 1.0f / ll;
      u16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = from_f32<T>(aa[e] * inv);
      const size_t at = packed ? packed_off(b, hq * D + cc * 8, (Hq * D) >> 5) : ((size_t)b * Hq + hq) * D + cc * 8;
      *reinterpret_cast<u16x8*>(out + at) = o;
    } else {
      float* p = part + (((size_t)b * Hq + hq) * S + split) * (D + 2);
      if (cc == 0) {
        p[0] = mm;
        p[1] = ll;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) p[2 + cc * 8 + e] = aa[e];
    }
  }
}

// ---------------------------------------------------------------------------------
// Grouped-query decode attention on the matrix cores.  With G >= 4 query heads per KV
// head the per-key dot products of the kernel above cost G times the vector work and
// it stops being memory-bound; here the G heads of a group form the (padded) 16
// columns of one MFMA tile, so a KV head's keys and values are read once for the whole
// group and the arithmetic moves to the matrix cores:
//   S^T = K Q^T    A = 16 key rows x 32 of d straight from the KV slice (rows chosen as
//                  keys 8*(r/4) + 4*t + r%4 so a lane ends up with 8 consecutive keys),
//                  B = Q^T of the group;
//   O^T = V^T P^T  A = V^T read from a per-wavefront LDS tile transposed while staged,
//                  B = P^T from registers; the head index stays on lane%16 for both.
// One workgroup = 4 wavefronts per (sequence, KV head, key range); each wavefront takes
// every 4th 32-key tile with its own online softmax; the four are merged lane-locally
// through LDS in fixed order.  Output format identical to the kernel above.
template <class T, int D, int G, bool FA>
__global__ __launch_bounds__(256) void attn_decode_gqa_kernel(
    const uint16_t* __restrict__ qkv, const uint16_t* __restrict__ kv, const int32_t* __restrict__ len_before,
    const int32_t* __restrict__ kv_off, const int32_t* __restrict__ cap, uint16_t* __restrict__ out,
    float* __restrict__ part, int Hq, int Hkv, int S, int packed, uint16_t* __restrict__ kvw,
    uint16_t* __restrict__ mirror, const float* __restrict__ inv_freq, int rope, QkvPlanes qp) {
  constexpr int LD = 40, DK = D / 32, DT = D / 16;
  constexpr int kVtWave = D * LD;                        // uint16 elements of one wavefront's V^T tile
  constexpr int kMrgLane = 2 + DT * 4;                   // floats a lane contributes to the merge
  static_assert(64 * kMrgLane * 4 <= kVtWave * 2, "merge buffer must fit the V^T tile");
  __shared__ __attribute__((aligned(16))) uint16_t smem[4 * kVtWave];
  __shared__ __attribute__((aligned(16))) uint16_t stage[FA ? G + 2 : 1][D];

  const int b = blockIdx.x / Hkv, hk = blockIdx.x % Hkv, split = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int len = len_before[b] + 1;
  const int chunk = (len + S - 1) / S;
  const int j0 = split * chunk, j1 = min(len, j0 + chunk);
  const int qkv_ld = (Hq + 2 * Hkv) * D;
  const bool qok = r < G;

  const int cp = cap[b];
  const size_t k_base = (size_t)kv_off[b] * 2 * Hkv * D + (size_t)(hk * 2) * cp * D;
  const int pos = len - 1;            // position of this step's token
  if (FA) {
    stage_new_token<T, D, G>(stage, qkv + (size_t)b * qkv_ld, qp, b, hk, Hq, Hkv, pos, inv_freq, rope);
    __syncthreads();
    if (pos >= j0 && pos < j1)
      store_new_token<D, G>(stage, kvw, mirror, k_base + (size_t)pos * D, k_base + ((size_t)cp + pos) * D);
  }
  u16x8 qf[DK];
#pragma unroll
  for (int kk = 0; kk < DK; ++kk) {
    qf[kk] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
    if (qok)
      qf[kk] = FA ? *reinterpret_cast<const u16x8*>(&stage[r][kk * 32 + g * 8])
                  : *reinterpret_cast<const u16x8*>(qkv + (size_t)b * qkv_ld + (size_t)(hk * G + r) * D + kk * 32 + g * 8);
  }
  const uint16_t* Kb = kv + k_base;
  const uint16_t* Vb = Kb + (size_t)cp * D;
  // last cached row a load may touch: with the fused append the new row is never loaded
  const int jlast = FA ? max(min(j1 - 1, pos - 1), 0) : j1 - 1;
  const float scale = rsqrtf((float)D);
  uint16_t* vt = smem + wave * kVtWave;

  float m = kNegBig, l = 0.f;
  f32x4 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int jt = j0 + wave * 32; jt < j1; jt += 4 * 32) {
    // stage V[jt..jt+32) transposed into this wavefront's LDS tile (wavefront-private: no workgroup barrier)
    // each lane takes (key pair, 8 d-values) items: two 16-byte loads, later eight 4-byte LDS writes
    constexpr int CH = 16 * (D / 8) / 64;                // items per lane
    u16x8 va[CH], vb[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int id = lane + 64 * c, key = 2 * (id & 15), dc = id >> 4;
      va[c] = vb[c] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
      const int ka = jt + key, kb = ka + 1;
      if (FA && ka == pos) va[c] = *reinterpret_cast<const u16x8*>(&stage[G + 1][dc * 8]);
      else if (ka < j1) va[c] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(Vb + (size_t)ka * D + dc * 8));
      if (FA && kb == pos) vb[c] = *reinterpret_cast<const u16x8*>(&stage[G + 1][dc * 8]);
      else if (kb < j1) vb[c] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(Vb + (size_t)kb * D + dc * 8));
    }
    f32x4 st[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      st[t] = f32x4{0.f, 0.f, 0.f, 0.f};
      const int key = jt + 8 * (r >> 2) + 4 * t + (r & 3);
      const uint16_t* kp = Kb + (size_t)min(key, jlast) * D + g * 8;        // clamped; masked below
      const bool fresh = FA && key == pos;
#pragma unroll
      for (int kk = 0; kk < DK; ++kk) {
        u16x8 kf = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(kp + kk * 32));
        if (fresh) kf = *reinterpret_cast<const u16x8*>(&stage[G][kk * 32 + g * 8]);
        st[t] = mma16x16x32<T>(kf, qf[kk], st[t]);
      }
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int id = lane + 64 * c, key = 2 * (id & 15), dc = id >> 4;
      const u16x8 ra = rot_pairs(va[c], g), rb = rot_pairs(vb[c], g);
#pragma unroll
      for (int e0 = 0; e0 < 8; ++e0) {
        const int e = (e0 + 2 * g) & 7;                  // the four 16-lane groups write different rows: fewer bank conflicts
        *reinterpret_cast<uint32_t*>(&vt[(dc * 8 + e) * LD + key]) = (uint32_t)ra[e0] | ((uint32_t)rb[e0] << 16);
      }
    }
    float sc[8], mx = kNegBig;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const bool ok = jt + 8 * g + e < j1;
      sc[e] = ok ? st[e >> 2][e & 3] * scale : kNegBig;
      mx = fmaxf(mx, sc[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float mn = fmaxf(m, mx);
    const float corr = __expf(m - mn);
    float rs = 0.f;
    u16x8 pb;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float p = sc[e] > 0.5f * kNegBig ? __expf(sc[e] - mn) : 0.f;
      rs += p;
      pb[e] = from_f32<T>(p);
    }
    l = l * corr + rs;
    m = mn;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the tile written above is read by other lanes below
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const u16x8 vf = *reinterpret_cast<const u16x8*>(&vt[(dt * 16 + r) * LD + g * 8]);
#pragma unroll
      for (int i = 0; i < 4; ++i) o[dt][i] *= corr;
      o[dt] = mma16x16x32<T>(vf, pb, o[dt]);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // reads done before the next trip overwrites the tile
    __builtin_amdgcn_wave_barrier();
  }

  // merge the four wavefronts lane by lane (same lane = same head and same d columns), in order
  __syncthreads();
  float* mrg = reinterpret_cast<float*>(smem);
  {
    float* mine = mrg + ((size_t)wave * 64 + lane) * kMrgLane;
    mine[0] = m;
    mine[1] = l;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i) mine[2 + dt * 4 + i] = o[dt][i];
  }
  __syncthreads();
  if (wave != 0) return;
  for (int w = 1; w < 4; ++w) {
    const float* other = mrg + ((size_t)w * 64 + lane) * kMrgLane;
    const float m2 = other[0], mn = fmaxf(m, m2);
    const float c1 = __expf(m - mn), c2 = __expf(m2 - mn);
    l = l * c1 + other[1] * c2;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i) o[dt][i] = o[dt][i] * c1 + other[2 + dt * 4 + i] * c2;
    m = mn;
  }
  l += __shfl_xor(l, 16, 64);
  l += __shfl_xor(l, 32, 64);
  if (!qok) return;
  const int hq = hk * G + r;
  if (S == 1) {
    const float inv = 1.0f / l;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      u16x4 w4;
#pragma unroll
      for (int i = 0; i < 4; ++i) w4[i] = from_f32<T>(o[dt][i] * inv);
      const int k = hq * D + dt * 16 + g * 4;
      const size_t at = packed ? packed_off(b, k, (Hq * D) >> 5) : (size_t)b * Hq * D + k;
      *reinterpret_cast<u16x4*>(out + at) = w4;
    }
  } else {
    float* p = part + (((size_t)b * Hq + hq) * S + split) * (D + 2);
    if (g == 0) {
      p[0] = m;
      p[1] = l;
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i) p[2 + dt * 16 + g * 4 + i] = o[dt][i];
  }
}

// ---------------------------------------------------------------------------------
// The same for head dimension 128, with every load instruction reading whole cache lines.
//
// In the kernel above a load instruction fetches the MFMA operand of 16 keys: 64 bytes from each of 16 rows.
// Half-line requests cost a fifth of the bandwidth (pure reads of this layout: 5.6 TB/s with that lane mapping,
// 7.1 TB/s with 4 whole 256-byte rows per instruction).  Here all loads are whole rows or whole lines and the
// operands are formed without LDS:
//   V: lane (x = lane % 16, y = lane / 16) loads, for i = 0..7, the 16 bytes d = 8x..8x+7 of key 8y+i -- four whole
//      rows per instruction.  It then holds an 8 x 8 block (keys x d); transposed in registers, row e of the block
//      is the B operand of product e of  O = P V:  B_e[key 8y+i][column x] = V[8y+i][8x+e], A = P[head][key] --
//      column x of product e is d = 8x + e, so the 8 products cover d = 0..127 and a lane ends up with 8 consecutive
//      d-values per head: one 16-byte store.
//   K: eight lanes share a key row (128 bytes = one line per instruction).  Lane x carries key x/2 of a set of 8
//      and the 64-byte half x%2 of a 128-byte part u of the row, so as an MFMA A operand "row x" is (key, half):
//      one product against Q's d-chunks of half 0 is right for the even rows, one against half 1 for the odd rows,
//      and a key's score is the sum of its even row of the first and its odd row of the second (the same lane
//      holds both).  Twice the matrix-core work for S, which has room to spare.  The keys of set s are
//      8y' + 2s + {0, 1} (y' = 0..3), so lane group y' ends up with scores of keys 8y'..8y'+7 -- the layout of
//      P as A operand and of V's rows as B operand.
// The rescale factor of the running softmax lives with the head on lane x; the accumulators hold heads 4y + j,
// so it is fetched across lanes (4 per tile).  Loads for the next tile are issued as soon as the registers of
// this one have been consumed: K after the score products, V after the output products.
template <class T, int G, bool FA>
__global__ __launch_bounds__(256, 2) void attn_decode_gqa128_kernel(
    const uint16_t* __restrict__ qkv, const uint16_t* __restrict__ kv, const int32_t* __restrict__ len_before,
    const int32_t* __restrict__ kv_off, const int32_t* __restrict__ cap, uint16_t* __restrict__ out,
    float* __restrict__ part, int Hq, int Hkv, int S, int packed, uint16_t* __restrict__ kvw,
    uint16_t* __restrict__ mirror, const float* __restrict__ inv_freq, int rope, QkvPlanes qp) {
  constexpr int D = 128;
  constexpr int NW = 4;                                  // wavefronts per workgroup (8 measured no better, even at one workgroup per CU)
  constexpr int kMrgWave = 32 + 16 * D;                  // floats per wavefront in the merge: m[16], l[16], O[16][D]
  __shared__ __attribute__((aligned(16))) float mrg[NW * kMrgWave];
  __shared__ __attribute__((aligned(16))) uint16_t stage[FA ? G + 2 : 1][D];

  const int b = blockIdx.x / Hkv, hk = blockIdx.x % Hkv, split = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int len = len_before[b] + 1;
  const int chunk = (len + S - 1) / S;
  const int j0 = split * chunk, j1 = min(len, j0 + chunk);
  const int qkv_ld = (Hq + 2 * Hkv) * D;
  const bool qok = r < G;

  const int cp = cap[b];
  const size_t k_base = (size_t)kv_off[b] * 2 * Hkv * D + (size_t)(hk * 2) * cp * D;
  const int pos = len - 1;            // position of this step's token
  if (FA) {
    stage_new_token<T, D, G>(stage, qkv + (size_t)b * qkv_ld, qp, b, hk, Hq, Hkv, pos, inv_freq, rope);
    __syncthreads();
    if (pos >= j0 && pos < j1)
      store_new_token<D, G>(stage, kvw, mirror, k_base + (size_t)pos * D, k_base + ((size_t)cp + pos) * D);
  }
  // B operands of the score products: Q[head r][32 kk + 8 g ..], zero for the padding heads
  u16x8 qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    qf[kk] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
    if (qok)
      qf[kk] = FA ? *reinterpret_cast<const u16x8*>(&stage[r][kk * 32 + g * 8])
                  : *reinterpret_cast<const u16x8*>(qkv + (size_t)b * qkv_ld + (size_t)(hk * G + r) * D + kk * 32 + g * 8);
  }
  const uint16_t* Kb = kv + k_base;
  const uint16_t* Vb = Kb + (size_t)cp * D;
  // last cached row a load may touch: with the fused append the new row is never loaded (the workgroup of the
  // range that owns it is writing it); rows past the end of the range are clamped to it and their scores masked
  const int jlast = FA ? max(min(j1 - 1, pos - 1), 0) : j1 - 1;
  const float scale = rsqrtf((float)D);

  // this lane's K rows: set s -> key offset 8 (r / 4) + 2 s + (r / 2) % 2, bytes 128 u + 64 (r % 2) + 16 g
  const int kkey = 8 * (r >> 2) + ((r >> 1) & 1);
  const int kcol = 32 * (r & 1) + 8 * g;
  u16x8 kreg[4][2], vreg[8];
  auto issue_k = [&](int jt) {
#pragma unroll
    for (int s2 = 0; s2 < 4; ++s2) {
      const uint16_t* kp = Kb + (size_t)min(jt + kkey + 2 * s2, jlast) * D + kcol;
#pragma unroll
      for (int u = 0; u < 2; ++u) kreg[s2][u] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(kp + 64 * u));
    }
  };
  auto issue_v = [&](int jt) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      vreg[i] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(Vb + (size_t)min(jt + 8 * g + i, jlast) * D + 8 * r));
  };

  float m = kNegBig, l = 0.f;
  f32x4 o[8];                         // o[e][j] = O[head 4 g + j][d = 8 r + e]
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  // The range is walked in rounds of NW tiles, one per wavefront (the workgroup reads NW * 8 KiB of K and of V side
  // by side).  A wavefront's tile of the last round may lie past the end: clamped loads, every score masked.
  // (Starting every workgroup at a different round was tried against the one stride at which all workgroups hit
  // the same memory channel in lock-step; it cost 3-9 % everywhere else, and the layout now avoids that stride.)
  const int nrounds = j1 > j0 ? (j1 - j0 + NW * 32 - 1) / (NW * 32) : 0;
  auto tile_at = [&](int i) { return j0 + (wave + NW * min(i, nrounds - 1)) * 32; };   // past the last round: that one again
  if (nrounds > 0) {
    issue_k(tile_at(0));
    issue_v(tile_at(0));
  }
  for (int ti = 0; ti < nrounds; ++ti) {
    const int jt = tile_at(ti), jnext = tile_at(ti + 1);
    const bool own = FA && pos >= jt && pos < jt + 32;   // the tile with this step's own token (wavefront-uniform)
    if (own) {
#pragma unroll
      for (int s2 = 0; s2 < 4; ++s2)
        if (jt + kkey + 2 * s2 == pos)
#pragma unroll
          for (int u = 0; u < 2; ++u) kreg[s2][u] = *reinterpret_cast<const u16x8*>(&stage[G][64 * u + kcol]);
    }
    // scores: keys jt + 8 g + e of head r
    float sc[8];
#pragma unroll
    for (int s2 = 0; s2 < 4; ++s2) {
      f32x4 d0 = f32x4{0.f, 0.f, 0.f, 0.f}, d1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        d0 = mma16x16x32<T>(kreg[s2][u], qf[2 * u], d0);
        d1 = mma16x16x32<T>(kreg[s2][u], qf[2 * u + 1], d1);
      }
      sc[2 * s2] = d0[0] + d1[1];
      sc[2 * s2 + 1] = d0[2] + d1[3];
    }
    __builtin_amdgcn_sched_barrier(0);
    issue_k(jnext);
    __builtin_amdgcn_sched_barrier(0);
    float mx = kNegBig;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      sc[e] = jt + 8 * g + e < j1 ? sc[e] * scale : kNegBig;
      mx = fmaxf(mx, sc[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float mn = fmaxf(m, mx);
    const float corr = __expf(m - mn);
    float rs = 0.f;
    u16x8 pb;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float p = sc[e] > 0.5f * kNegBig ? __expf(sc[e] - mn) : 0.f;
      rs += p;
      pb[e] = from_f32<T>(p);
    }
    l = l * corr + rs;
    m = mn;
    float cj[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) cj[j] = __shfl(corr, 4 * g + j, 64);
    if (own) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (jt + 8 * g + i == pos) vreg[i] = *reinterpret_cast<const u16x8*>(&stage[G + 1][8 * r]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      // row e of the transposed 8 x 8 block: d = 8 r + e of keys 8 g .. 8 g + 7
      u32x4 bw;
#pragma unroll
      for (int i2 = 0; i2 < 4; ++i2) {
        const uint32_t lo = __builtin_bit_cast(u32x4, vreg[2 * i2])[e >> 1], hi = __builtin_bit_cast(u32x4, vreg[2 * i2 + 1])[e >> 1];
        bw[i2] = (e & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) o[e][j] *= cj[j];
      o[e] = mma16x16x32<T>(pb, __builtin_bit_cast(u16x8, bw), o[e]);
    }
    __builtin_amdgcn_sched_barrier(0);
    issue_v(jnext);
    __builtin_amdgcn_sched_barrier(0);
  }
  l += __shfl_xor(l, 16, 64);
  l += __shfl_xor(l, 32, 64);

  // merge the NW wavefronts through LDS, in order: per head m, l; per (head, d) the accumulators
  float* mine = mrg + (size_t)wave * kMrgWave;
  if (g == 0) {
    mine[r] = m;
    mine[16 + r] = l;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float* row = mine + 32 + (size_t)(4 * g + j) * D + 8 * r;
    *reinterpret_cast<f32x4*>(row) = f32x4{o[0][j], o[1][j], o[2][j], o[3][j]};
    *reinterpret_cast<f32x4*>(row + 4) = f32x4{o[4][j], o[5][j], o[6][j], o[7][j]};
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int h = 4 * g + j;
    if (h >= G) continue;
    float mm = mrg[h], ll = mrg[16 + h];
    float acc[8];
    {
      const float* row = mrg + 32 + (size_t)h * D + 8 * r;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = row[e];
    }
    for (int w = 1; w < NW; ++w) {
      const float* other = mrg + (size_t)w * kMrgWave;
      const float m2 = other[h], mn = fmaxf(mm, m2);
      const float c1 = __expf(mm - mn), c2 = __expf(m2 - mn);
      ll = ll * c1 + other[16 + h] * c2;
      const float* row = other + 32 + (size_t)h * D + 8 * r;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = acc[e] * c1 + row[e] * c2;
      mm = mn;
    }
    const int hq = hk * G + h;
    if (S == 1) {
      const float inv = 1.0f / ll;
      u16x8 w8;
#pragma unroll
      for (int e = 0; e < 8; ++e) w8[e] = from_f32<T>(acc[e] * inv);
      const int k = hq * D + 8 * r;
      const size_t at = packed ? packed_off(b, k, (Hq * D) >> 5) : (size_t)b * Hq * D + k;
      *reinterpret_cast<u16x8*>(out + at) = w8;
    } else {
      float* p = part + (((size_t)b * Hq + hq) * S + split) * (D + 2);
      if (r == 0) {
        p[0] = mm;
        p[1] = ll;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) p[2 + 8 * r + e] = acc[e];
    }
  }
}

// Merge the S key-range partials of one (sequence, query head); thread = output element.
template <class T, int D>
__global__ void attn_combine_kernel(const float* __restrict__ part, uint16_t* __restrict__ out, int S, int Hq,
                                    int packed) {
  const float* p = part + (size_t)blockIdx.x * S * (D + 2);
  const int e = threadIdx.x;
  float mx = kNegBig;
  for (int s = 0; s < S; ++s) mx = fmaxf(mx, p[(size_t)s * (D + 2)]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < S; ++s) {
    const float w = __expf(p[(size_t)s * (D + 2)] - mx);
    den += w * p[(size_t)s * (D + 2) + 1];
    num += w * p[(size_t)s * (D + 2) + 2 + e];
  }
  const int b = blockIdx.x / Hq, hq = blockIdx.x % Hq;
  const size_t at = packed ? packed_off(b, hq * D + e, (Hq * D) >> 5) : (size_t)blockIdx.x * D + e;
  out[at] = from_f32<T>(num / den);
}

// Key-range splits: one workgroup per CU (256) is enough once each keeps 64 KiB in
// flight; below that, split the keys, at least 256 per split, at most 16 splits.
int attn_decode_splits(int B, int Hkv, int max_len) {
  const int pairs = B * Hkv;
  int S = (256 + pairs - 1) / pairs;
  const int by_len = (max_len + 255) / 256;
  if (S > by_len) S = by_len;
  if (S > 16) S = 16;
  if (S < 1) S = 1;
  return S;
}

template <class T, int D, bool FA>
static hipError_t launch_d(const uint16_t* qkv, const uint16_t* kv, const StepIndex& ix, uint16_t* out,
                           float* part, int B, int Hq, int Hkv, int S, int packed, const AttnAppend& ap,
                           hipStream_t st) {
  const int G = Hq / Hkv;
  const QkvPlanes qp{FA ? ap.qkv_part : nullptr, ap.qkv_nsplit, ap.qkv_rows};
#define SN_LAUNCH_G(GV, NWV, UKV)                                                                                 \
  SN_LAUNCH((attn_decode_kernel<T, D, GV, NWV, UKV, FA>), dim3(B * Hkv, S), dim3(NWV * 64), 0, st, qkv, kv,       \
            ix.len_before, ix.kv_off, ix.cap, out, part, Hq, Hkv, S, packed, ap.kv, ap.mirror, ap.inv_freq, ap.rope, qp)
#define SN_LAUNCH_GQA(GV)                                                                                         \
  if constexpr (D == 128)                                                                                         \
    SN_LAUNCH((attn_decode_gqa128_kernel<T, GV, FA>), dim3(B * Hkv, S), dim3(256), 0, st, qkv, kv, ix.len_before, \
              ix.kv_off, ix.cap, out, part, Hq, Hkv, S, packed, ap.kv, ap.mirror, ap.inv_freq, ap.rope, qp);      \
  else                                                                                                            \
    SN_LAUNCH((attn_decode_gqa_kernel<T, D, GV, FA>), dim3(B * Hkv, S), dim3(256), 0, st, qkv, kv, ix.len_before, \
              ix.kv_off, ix.cap, out, part, Hq, Hkv, S, packed, ap.kv, ap.mirror, ap.inv_freq, ap.rope, qp)
  switch (G) {
    // head dimension 128: the whole-line matrix-core kernel also for one or two query heads per KV head (15 of its
    // 16 columns idle, but the bound is the memory system: 32 x 40 heads x 1030 keys 113 -> 103 us, 8 x 32 x 530
    // 16.2 -> 13.8 us against the vector kernel)
    case 1:
      if constexpr (D == 128) { SN_LAUNCH_GQA(1); } else { SN_LAUNCH_G(1, 16, 2); }
      break;
    case 2:
      if constexpr (D == 128) { SN_LAUNCH_GQA(2); } else { SN_LAUNCH_G(2, 16, 2); }
      break;
    case 4: SN_LAUNCH_GQA(4); break;
    case 8: SN_LAUNCH_GQA(8); break;
    default: return hipErrorInvalidValue;
  }
#undef SN_LAUNCH_G
#undef SN_LAUNCH_GQA
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || S == 1) return e;
  SN_LAUNCH((attn_combine_kernel<T, D>), dim3(B * Hq), dim3(D), 0, st, part, out, S, Hq, packed);
  return hipGetLastError();
}

hipError_t launch_attn_decode(int dtype, const void* qkv16, const void* kv, const StepIndex& ix, void* out16,
                              float* part, int B, int Hq, int Hkv, int d, int S, hipStream_t st, int packed,
                              const AttnAppend* append) {
  if (B <= 0) return hipSuccess;
  const uint16_t* q = (const uint16_t*)qkv16;
  const uint16_t* k = (const uint16_t*)kv;
  uint16_t* o = (uint16_t*)out16;
  if (append && (!append->kv || (append->rope && !append->inv_freq))) return hipErrorInvalidValue;
  if (append && append->qkv_part && (append->qkv_nsplit < 1 || append->qkv_nsplit > kMaxSplits || append->qkv_rows < B))
    return hipErrorInvalidValue;
  if (!q && !(append && append->qkv_part)) return hipErrorInvalidValue;
  const AttnAppend ap = append ? *append : AttnAppend{};
#define SN_DISPATCH(TT, DD)                                                                        \
  return append ? launch_d<TT, DD, true>(q, k, ix, o, part, B, Hq, Hkv, S, packed, ap, st)         \
                : launch_d<TT, DD, false>(q, k, ix, o, part, B, Hq, Hkv, S, packed, ap, st)
  if (dtype == 0) {
    if (d == 64) SN_DISPATCH(F16, 64);
    if (d == 128) SN_DISPATCH(F16, 128);
  } else {
    if (d == 64) SN_DISPATCH(BF16, 64);
    if (d == 128) SN_DISPATCH(BF16, 128);
  }
#undef SN_DISPATCH
  return hipErrorInvalidValue;
}

}  // namespace sn
