// Host-callable launchers of the gfx950 layer kernels.  Every launcher enqueues on
// the given stream and returns the hipError_t of the launch.  Launch geometry depends
// only on sizes, never on pointer values, so the same inputs give the same bits
// whether a layer's state sits in a resident buffer or in a staging slot.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sn {

// Optional timing of the NEXT kernel launch on this host thread: when start/stop are
// set, the launch records the kernel's own begin and end timestamps into them (no
// extra marker packets on the stream) and clears the pair.
struct LaunchEvents {
  hipEvent_t start = nullptr, stop = nullptr;
};
LaunchEvents& next_launch_events();

enum Epilogue {
  EPI_STORE16 = 0,   // out16[m][n] = acc + bias
  EPI_GELU16 = 1,    // out16[m][n] = gelu(acc + bias)
  EPI_RESID32 = 2,   // x32[m][n] += acc + bias
  EPI_SWIGLU16 = 3,  // weights hold gate/up in alternating 16-row blocks: out16[m][n] = silu(g)*u
  EPI_PART32 = 4     // split-K: part[split][m][n] = partial product (no bias); folded in by the consumer
};
constexpr int kMaxSplits = 8;
constexpr int kMaxDecodeRows = 128;  // most token rows of a decode step (the weight-streaming projections)
constexpr int kPrefillQTile = 128;   // query rows (new tokens of one sequence) per prefill-attention workgroup

// Pending split-K partial sums of a residual projection: the next kernel that reads the
// residual stream first performs x32[m][n] += bias[n] + sum_s part[s][m][n] (s ascending).
struct Fold {
  const float* part = nullptr;   // [nsplit][T][h]
  int nsplit = 0;
  const void* bias = nullptr;    // 16-bit [h] or null
};

// Per-iteration index arrays (device int32), built on the host by sn_step.
struct StepIndex {
  const int32_t* len_before;  // [B] tokens cached before this iteration
  const int32_t* n_new;       // [B]
  const int32_t* tok_start;   // [B] first row of the sequence in the token-major buffers
  const int32_t* kv_off;      // [B] token offset of the sequence inside a layer's KV slice
  const int32_t* cap;         // [B] KV capacity of the sequence (tokens)
  const int32_t* tok_seq;     // [T] sequence of each token row
  const int32_t* tok_pos;     // [T] absolute position of each token row
  const int32_t* tile_seq;    // [n_qtiles] prefill attention: sequence of each kPrefillQTile-row query tile
  const int32_t* tile_q0;     // [n_qtiles] first new-token index of the tile inside its sequence
};

// flag (device int32, may be null): launch_cast_in clears it, the output casts set it to 1 when a hidden state is inf or NaN.
hipError_t launch_cast_in(int dtype, const void* in16, float* x32, size_t n, hipStream_t st, int32_t* flag = nullptr);
hipError_t launch_cast_out(int dtype, const float* x32, void* out16, size_t n, hipStream_t st, int32_t* flag = nullptr);
// Same after folding pending partial sums into x32 (written back); bias_dtype: type of fold.bias.
hipError_t launch_cast_out_fold(int dtype, int bias_dtype, float* x32, void* out16, int T, int h, const Fold& fold,
                                hipStream_t st, int32_t* flag = nullptr);
hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
// Debug aids: fill `bytes` (multiple of 16) with a 32-bit pattern; keep a stream busy for `ticks` wall-clock
// periods (bounded by max_trips sleeps of a few microseconds each, so the kernel always ends).
hipError_t launch_fill(void* dst, size_t bytes, uint32_t pattern, hipStream_t st);
hipError_t launch_delay(uint64_t ticks, int max_trips, hipStream_t st);
hipError_t launch_fill_hash(int dtype, void* out16, size_t n, uint32_t seed, hipStream_t st);

// u16[t][:] = norm(x32[t][:]) * gain (+ shift); shift == nullptr for RMSNorm.
hipError_t launch_norm(int dtype, int is_ln, const float* x32, const void* gain, const void* shift,
                       void* u16, int T, int h, float eps, hipStream_t st);
// Same, after folding pending partial sums into x32 (x32 is updated in place).
hipError_t launch_norm_fold(int dtype, int is_ln, float* x32, const void* gain, const void* shift, void* u16, int T,
                            int h, float eps, const Fold& fold, hipStream_t st, int packed_out = 0);

// out = epilogue(X[M][K] * W^T), W tiled [N/16][K/32][64][8].  N counts weight rows
// (2*ffn for EPI_SWIGLU16, whose output has N/2 columns).  Decode path: M <= kMaxDecodeRows.
// flags: kXPacked -- X is row-tile packed (common.h packed_off); kOutPacked -- the 16-bit
// output is written row-tile packed (it feeds the next decode projection).
constexpr int kXPacked = 1, kOutPacked = 2;
hipError_t launch_gemm_skinny(int dtype, int epi, const void* W, const void* X, const void* bias,
                              void* out, int M, int N, int K, hipStream_t st, int splits = 1, int flags = 0);
int gemm_skinny_splits(int M, int N, int K);
// Planes for a QKV projection run as EPI_PART32 (summed by the attention kernel, AttnAppend::qkv_part), or 0:
// keep the 16-bit epilogue.  Non-zero only at 9..128 rows, where the split shape is the faster one.
int gemm_qkv_splits(int M, int N, int K);
// Prefill path: any M.
hipError_t launch_gemm_tile(int dtype, int epi, const void* W, const void* X, const void* bias,
                            void* out, int M, int N, int K, hipStream_t st, int flags = 0);
bool gemm_tile_takes_packed(int M, int N, int K);   // the 256 x 256 kernel applies: flags kXPacked / kOutPacked allowed

// Rotates q (in place) and k, and appends k, v rows to the layer's KV slice
// ([seq][Hkv][K|V][cap][d]); mirror (may be null) is a second copy of the slice that
// receives the same rows (host-resident master of an offloaded layer).  k and v are
// rounded to kv_value_dtype before being stored in containers of type dtype
// (allowed pairs: f16/f16, f16/bf16, bf16/bf16).
hipError_t launch_rope_append(int dtype, int kv_value_dtype, void* qkv16, const StepIndex& ix, void* kv,
                              void* mirror, const float* inv_freq, int T, int Hq, int Hkv, int d, int rope,
                              hipStream_t st);

// One query per sequence over len_before+1 cached keys.  part: fp32 scratch for
// split partials, [B][Hq][S][d+2].  append == nullptr: the new row is already in the KV
// slice and q, k are already rotated.  Otherwise the kernel does that itself: it rotates
// q and k of row b of qkv16 (when rope != 0), stores k, v at position len_before[b] of
// the slice `kv` (and of `mirror`, if not null) and attends over them from registers.
struct AttnAppend {
  uint16_t* kv = nullptr;
  uint16_t* mirror = nullptr;
  const float* inv_freq = nullptr;
  int rope = 0;
  // the step's q, k, v as split-K partial planes [qkv_nsplit][qkv_rows][(Hq + 2 Hkv) d] (bias in plane 0)
  // instead of the 16-bit qkv rows; null: read qkv16
  const float* qkv_part = nullptr;
  int qkv_nsplit = 0;
  int qkv_rows = 0;
};
int attn_decode_splits(int B, int Hkv, int max_len);
hipError_t launch_attn_decode(int dtype, const void* qkv16, const void* kv, const StepIndex& ix,
                              void* out16, float* part, int B, int Hq, int Hkv, int d, int S,
                              hipStream_t st, int packed_out = 0, const AttnAppend* append = nullptr);
// Causal attention of each sequence's new tokens over its cached + new keys.
hipError_t launch_attn_prefill(int dtype, const void* qkv16, const void* kv, const StepIndex& ix,
                               void* out16, int n_qtiles, int Hq, int Hkv, int d, hipStream_t st, int packed = 0);

}  // namespace sn
