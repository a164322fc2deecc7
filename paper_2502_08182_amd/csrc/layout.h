// Byte layouts: the caller-side layer blob (plain row-major tensors) and the
// library's own per-layer record, in which every matrix is stored as 16x32 tiles in
// the lane order of the gfx950 16x16x32 matrix-core instruction, so that a wavefront
// reads one tile as 64 consecutive 16-byte pieces.
#pragma once
#include <stdint.h>

#include "../../include/sn.h"

namespace sn {

constexpr uint64_t kAlign = 256;
inline uint64_t align_up(uint64_t v, uint64_t a = kAlign) { return (v + a - 1) / a * a; }

// Offsets (bytes) into the caller-side blob; ~0 where the tensor does not exist.
struct BlobLayout {
  uint64_t wqkv, bqkv, wo, bo, wg, bg, wu, bu, wd, bd, n1g, n1b, n2g, n2b, total;
};
constexpr uint64_t kNone = ~0ull;
BlobLayout blob_layout(const sn_model_shape& s);

// Offsets (bytes) into the library's tiled layer record.
struct PackedLayout {
  uint64_t wqkv, wo, wup, wd;               // tiled matrices
  uint64_t bqkv, bo, bup, bd;               // vectors (kNone if has_bias == 0); bup: [bg | bu] for SwiGLU
  uint64_t n1g, n1b, n2g, n2b;              // norm parameters (n?b kNone for RMSNorm)
  uint64_t total;                           // multiple of kAlign
  int32_t n_qkv, n_up;                      // output widths: (Hq+2Hkv)*d ; ffn or 2*ffn (gate/up interleaved)
};
PackedLayout packed_layout(const sn_model_shape& s);

// Validate divisibility the kernels rely on; returns nullptr or a message.
const char* check_shape(const sn_model_shape& s);

// src: [N][K] row-major 16-bit; dst: tiles [N/16][K/32][64 lanes][8], lane = n%16 + 16*((k%32)/8).
// row_block_stride / row_block_offset place source block j at destination block
// j*row_block_stride + row_block_offset (2,0 / 2,1 interleave gate and up).
// bf16_to_f16: source elements are bfloat16 and are stored as the equal float16 value.
// Returns the number of elements that float16 cannot hold (|v| > 65504, inf, NaN).
uint64_t tile_matrix(uint16_t* dst, const uint16_t* src, int N, int K, int row_block_stride,
                     int row_block_offset, bool bf16_to_f16 = false);

// bfloat16 bits -> float16 bits of the same value.  Exact for 2^-17 <= |v| <= 65504 and 0;
// smaller magnitudes round to the nearest float16 subnormal (absolute error < 2^-25);
// *bad is incremented when the value is not representable (overflow, inf, NaN).
uint16_t bf16_bits_to_f16_bits(uint16_t b, uint64_t* bad);

// Caller blob -> tiled record (all 16-bit data stored as float16, the compute type).
// Returns the number of unrepresentable elements (0 on success).
uint64_t pack_layer(const sn_model_shape& s, const uint8_t* blob, uint8_t* record);

}  // namespace sn
