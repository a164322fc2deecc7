#include "layout.h"

#include <cstring>
#include <thread>
#include <vector>

namespace sn {

static uint64_t take(uint64_t& off, uint64_t elems) {
  const uint64_t at = off;
  off += align_up(elems * 2);
  return at;
}

BlobLayout blob_layout(const sn_model_shape& s) {
  BlobLayout b;
  const uint64_t h = s.hidden, F = s.ffn, qd = (uint64_t)s.n_q_heads * s.head_dim;
  const uint64_t nq = (uint64_t)(s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim;
  const bool bias = s.has_bias != 0, glu = s.act == SN_ACT_SWIGLU, ln = s.norm == SN_NORM_LN;
  uint64_t off = 0;
  b.wqkv = take(off, nq * h);
  b.bqkv = bias ? take(off, nq) : kNone;
  b.wo = take(off, h * qd);
  b.bo = bias ? take(off, h) : kNone;
  b.wg = glu ? take(off, F * h) : kNone;
  b.bg = (glu && bias) ? take(off, F) : kNone;
  b.wu = take(off, F * h);
  b.bu = bias ? take(off, F) : kNone;
  b.wd = take(off, h * F);
  b.bd = bias ? take(off, h) : kNone;
  b.n1g = take(off, h);
  b.n1b = ln ? take(off, h) : kNone;
  b.n2g = take(off, h);
  b.n2b = ln ? take(off, h) : kNone;
  b.total = off;
  return b;
}

PackedLayout packed_layout(const sn_model_shape& s) {
  PackedLayout p;
  const uint64_t h = s.hidden, F = s.ffn, qd = (uint64_t)s.n_q_heads * s.head_dim;
  const bool bias = s.has_bias != 0, glu = s.act == SN_ACT_SWIGLU, ln = s.norm == SN_NORM_LN;
  p.n_qkv = (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim;
  p.n_up = glu ? 2 * s.ffn : s.ffn;
  uint64_t off = 0;
  p.wqkv = take(off, (uint64_t)p.n_qkv * h);
  p.wo = take(off, h * qd);
  p.wup = take(off, (uint64_t)p.n_up * h);
  p.wd = take(off, h * F);
  p.bqkv = bias ? take(off, p.n_qkv) : kNone;
  p.bo = bias ? take(off, h) : kNone;
  p.bup = bias ? take(off, p.n_up) : kNone;
  p.bd = bias ? take(off, h) : kNone;
  p.n1g = take(off, h);
  p.n1b = ln ? take(off, h) : kNone;
  p.n2g = take(off, h);
  p.n2b = ln ? take(off, h) : kNone;
  p.total = off;
  return p;
}

const char* check_shape(const sn_model_shape& s) {
  if (s.n_layers < 1 || s.hidden < 32 || s.n_q_heads < 1 || s.n_kv_heads < 1 || s.ffn < 32)
    return "shape: non-positive dimension";
  if (s.head_dim != 64 && s.head_dim != 128) return "shape: head_dim must be 64 or 128";
  if (s.n_q_heads % s.n_kv_heads) return "shape: n_q_heads must be a multiple of n_kv_heads";
  if (s.n_q_heads / s.n_kv_heads > 8) return "shape: at most 8 query heads per KV head";
  if (s.hidden % 32 || s.ffn % 32) return "shape: hidden and ffn must be multiples of 32";
  if (s.hidden > 16384) return "shape: hidden above 16384 not supported";
  if (s.act != SN_ACT_GELU && s.act != SN_ACT_SWIGLU) return "shape: act";
  if (s.norm != SN_NORM_LN && s.norm != SN_NORM_RMS) return "shape: norm";
  if (s.dtype != SN_F16 && s.dtype != SN_BF16) return "shape: dtype";
  if (s.max_batch < 1 || s.max_seq < 1 || s.max_tokens < 0) return "shape: max_batch/max_seq/max_tokens";
  if (!(s.norm_eps >= 0.f) || !(s.rope_theta > 0.f)) return "shape: norm_eps/rope_theta";
  return nullptr;
}

uint16_t bf16_bits_to_f16_bits(uint16_t b, uint64_t* bad) {
  const uint32_t sign = (b & 0x8000u);
  const int e = (b >> 7) & 0xff;            // bfloat16: 8 exponent bits (bias 127), 7 mantissa bits
  const uint32_t m = b & 0x7fu;
  if (e == 0xff) {                          // inf / NaN
    if (bad) ++*bad;
    return (uint16_t)(sign | 0x7c00u | (m ? 0x200u : 0));
  }
  if (e == 0) return (uint16_t)sign;        // zero and bfloat16 subnormals (< 2^-126): zero in float16
  const int E = e - 127;                    // value = 1.m * 2^E
  if (E > 15) {
    if (bad) ++*bad;
    return (uint16_t)(sign | 0x7c00u);
  }
  if (E >= -14) return (uint16_t)(sign | (uint32_t)(E + 15) << 10 | m << 3);   // normal: exact
  // float16 subnormal: value = k * 2^-24 with k = round(1.m * 2^(E+24)), ties to even
  const int shift = -E - 17;                // (0x80|m) is 1.m * 2^7; k = (0x80|m) * 2^(E+17)
  const uint32_t sig = 0x80u | m;
  if (shift <= 0) return (uint16_t)(sign | (sig << -shift));
  if (shift > 9) return (uint16_t)sign;
  const uint32_t k = sig >> shift, rem = sig & ((1u << shift) - 1), half = 1u << (shift - 1);
  return (uint16_t)(sign | (k + ((rem > half || (rem == half && (k & 1))) ? 1 : 0)));
}

uint64_t tile_matrix(uint16_t* dst, const uint16_t* src, int N, int K, int row_block_stride,
                     int row_block_offset, bool bf16_to_f16) {
  const int NB = N / 16, KB = K / 32;
  const int nthreads = (uint64_t)N * K >= (1u << 22) ? 8 : 1;
  std::vector<uint64_t> bad(nthreads, 0);
  auto work = [&](int nb0, int nb1, int tid) {
    for (int nb = nb0; nb < nb1; ++nb) {
      uint16_t* out = dst + (uint64_t)(nb * row_block_stride + row_block_offset) * KB * 512;
      for (int kb = 0; kb < KB; ++kb) {
        for (int lane = 0; lane < 64; ++lane) {
          const uint16_t* in = src + (uint64_t)(nb * 16 + (lane & 15)) * K + kb * 32 + (lane >> 4) * 8;
          uint16_t* o = out + ((uint64_t)kb * 64 + lane) * 8;
          if (bf16_to_f16)
            for (int e = 0; e < 8; ++e) o[e] = bf16_bits_to_f16_bits(in[e], &bad[tid]);
          else
            std::memcpy(o, in, 16);
        }
      }
    }
  };
  if (nthreads == 1) {
    work(0, NB, 0);
    return bad[0];
  }
  std::vector<std::thread> pool;
  const int per = (NB + nthreads - 1) / nthreads;
  for (int t = 0; t < nthreads; ++t) {
    const int a = t * per, b = a + per < NB ? a + per : NB;
    if (a < b) pool.emplace_back(work, a, b, t);
  }
  for (auto& th : pool) th.join();
  uint64_t tot = 0;
  for (uint64_t v : bad) tot += v;
  return tot;
}

uint64_t pack_layer(const sn_model_shape& s, const uint8_t* blob, uint8_t* rec) {
  const BlobLayout b = blob_layout(s);
  const PackedLayout p = packed_layout(s);
  const int h = s.hidden, F = s.ffn, qd = s.n_q_heads * s.head_dim;
  const bool cv = s.dtype == SN_BF16;
  uint64_t bad = 0;
  auto src = [&](uint64_t off) { return reinterpret_cast<const uint16_t*>(blob + off); };
  auto dst = [&](uint64_t off) { return reinterpret_cast<uint16_t*>(rec + off); };
  bad += tile_matrix(dst(p.wqkv), src(b.wqkv), p.n_qkv, h, 1, 0, cv);
  bad += tile_matrix(dst(p.wo), src(b.wo), h, qd, 1, 0, cv);
  if (s.act == SN_ACT_SWIGLU) {
    bad += tile_matrix(dst(p.wup), src(b.wg), F, h, 2, 0, cv);
    bad += tile_matrix(dst(p.wup), src(b.wu), F, h, 2, 1, cv);
  } else {
    bad += tile_matrix(dst(p.wup), src(b.wu), F, h, 1, 0, cv);
  }
  bad += tile_matrix(dst(p.wd), src(b.wd), h, F, 1, 0, cv);
  auto vec = [&](uint64_t to, uint64_t from, uint64_t n) {
    if (to == kNone || from == kNone) return;
    if (!cv) {
      std::memcpy(rec + to, blob + from, n * 2);
      return;
    }
    const uint16_t* in = src(from);
    uint16_t* out = dst(to);
    for (uint64_t i = 0; i < n; ++i) out[i] = bf16_bits_to_f16_bits(in[i], &bad);
  };
  vec(p.bqkv, b.bqkv, p.n_qkv);
  vec(p.bo, b.bo, h);
  if (p.bup != kNone) {
    if (s.act == SN_ACT_SWIGLU) {
      vec(p.bup, b.bg, F);
      vec(p.bup + (uint64_t)F * 2, b.bu, F);
    } else {
      vec(p.bup, b.bu, F);
    }
  }
  vec(p.bd, b.bd, h);
  vec(p.n1g, b.n1g, h);
  vec(p.n1b, b.n1b, h);
  vec(p.n2g, b.n2g, h);
  vec(p.n2b, b.n2b, h);
  return bad;
}

}  // namespace sn
