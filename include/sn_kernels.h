/*
 * sn_kernels.h -- C ABI of the individual layer kernels (gfx950), one entry per step of
 * the decoder layer (paper Sec. 2.1: attention computations, then MLP computations), so
 * that each step can be checked against the oracle on its own.  sn_step (sn.h) launches
 * exactly these kernels.  All pointers are device pointers unless marked host; `stream`
 * is a hipStream_t passed as void*.  Return value: 0 or a negative SN_E_* code.
 * dtype: SN_F16 / SN_BF16 for all 16-bit buffers.
 */
#ifndef SN_KERNELS_H_
#define SN_KERNELS_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Host only: re-tile a row-major [N][K] 16-bit matrix (N % 16 == 0, K % 32 == 0) into
 * the 16x32-tile order the GEMM kernels read: tile (nb, kb) at (nb*K/32 + kb)*512
 * elements, element (n, k) of the tile at ((n%16) + 16*((k%32)/8))*8 + k%8.
 * dst_row_block_stride / offset: source block j lands at block j*stride + offset
 * (2,0 and 2,1 interleave a gate and an up matrix for the SwiGLU epilogue).
 * bf16_to_f16 != 0: the source holds bfloat16 values, the destination receives the same
 * values as float16 (exact for 2^-17 <= |v| <= 65504; smaller ones round to float16
 * subnormals).  Returns the number of elements float16 cannot hold (overflow, inf, NaN),
 * or a negative SN_E_* code. */
int64_t sn_k_tile_weights(const void* host_src, void* host_dst, int32_t N, int32_t K,
                          int32_t dst_row_block_stride, int32_t dst_row_block_offset,
                          int32_t bf16_to_f16);

/* Row-tile packed activations (decode path).  An [M][K] 16-bit activation matrix can be
 * stored in 16-row x 32-column tiles in matrix-core operand order, so that the decode
 * projections read it in 1 KiB pieces: element (m, k) sits at element offset
 *   (((m/16)*(K/32) + k/32)*64 + (m%16) + 16*((k%32)/8))*8 + k%8      (K % 32 == 0),
 * and a buffer holds 16*ceil(M/16) rows.  sn_k_packed_offset returns that offset (host
 * only).  Kernels take a flag where they can read or write this layout. */
uint64_t sn_k_packed_offset(int32_t m, int32_t k, int32_t K);

/* out16[t][:] = normalise(x32[t][:]) * gain (+ shift).  is_ln: LayerNorm (biased
 * variance) else RMSNorm (shift ignored).  x32 fp32 [T][h]; gain/shift 16-bit [h]. */
int sn_k_norm(int32_t dtype, int32_t is_ln, const void* x32, const void* gain, const void* shift,
              void* out16, int32_t T, int32_t h, float eps, void* stream);

/* out = epilogue(X[M][K] * W^T + bias), W tiled as above with N rows, bias 16-bit or NULL.
 * epilogue 0: 16-bit store; 1: GELU (erf) then 16-bit store; 2: out is the fp32 residual
 * stream [M][N], updated in place (+=); 3: SwiGLU -- W holds gate and up in alternating
 * 16-row blocks (N = 2*ffn rows), bias = [gate | up], out16[M][N/2] = silu(g)*u.
 * path 0: weight-streaming decode kernel (M <= 128; a packed X holds 16*ceil(M/16) rows); path 1: tiled prefill kernel.
 * flags: 1 = X is row-tile packed; 2 = the 16-bit output (epilogues 0, 1, 3) is written row-tile packed.
 * Path 1 takes them only where its 256 x 256 kernel applies (N % 256 == 0, K % 256 == 0, M > 128) and returns SN_E_INVAL otherwise: same values bit for bit, whole cache lines per
 * activation request instead of half ones. */
int sn_k_gemm(int32_t dtype, int32_t epilogue, int32_t path, const void* W, const void* X,
              const void* bias, void* out, int32_t M, int32_t N, int32_t K, int32_t flags,
              void* stream);

/* Decode-phase residual projection with the K dimension split over `splits` workgroup
 * ranges (1..8; 0: the library's choice): part[s][M][N] (fp32, device) receives the
 * partial product of range s; plane 0 also receives the bias (16-bit [N], may be NULL),
 * so that whoever folds the planes later needs nothing from this layer's weight record.
 * The consumer folds them into the residual stream in ascending s (sn_k_norm_fold,
 * sn_k_cast_out_fold), which keeps the sum order fixed.  flags: 1 = X is row-tile packed (what
 * a decode step passes).  Returns the number of splits used (> 0) or a negative SN_E_* code. */
int sn_k_gemm_splitk(int32_t dtype, const void* W, const void* X, const void* bias, void* part, int32_t M,
                     int32_t N, int32_t K, int32_t splits, int32_t flags, void* stream);

/* sn_k_norm preceded by x32[t][:] += bias + sum_s part[s][t][:] (x32 is updated in place;
 * bias 16-bit [h] or NULL; splits == 0: plain sn_k_norm).  packed_out != 0: out16 is
 * written row-tile packed. */
int sn_k_norm_fold(int32_t dtype, int32_t is_ln, void* x32, const void* gain, const void* shift,
                   void* out16, int32_t T, int32_t h, float eps, const void* part, int32_t splits,
                   const void* bias, int32_t packed_out, void* stream);

/* The same fold followed by the fp32 -> 16-bit output cast (x32 updated in place). */
int sn_k_cast_out_fold(int32_t dtype, void* x32, void* out16, int32_t T, int32_t h, const void* part,
                       int32_t splits, const void* bias, void* stream);

/* Index arrays shared by the attention-side kernels (device int32):
 *   len_before[B], n_new[B], tok_start[B], kv_off[B] (token offset of the sequence in the
 *   KV slice), cap[B]; tok_seq[T], tok_pos[T]; tile_seq[n_qtiles], tile_q0[n_qtiles].
 *   A query tile is a run of up to SN_K_PREFILL_QTILE consecutive new tokens of one sequence:
 *   tile_seq its sequence, tile_q0 the index of its first token among the sequence's new
 *   tokens (a multiple of SN_K_PREFILL_QTILE); every new token lies in exactly one tile.
 * KV slice layout: for sequence b at element offset kv_off[b]*2*Hkv*d:
 *   [Hkv][2 (K then V)][cap[b]][d], 16-bit. */

/* Rotate q (in place in qkv16 [T][(Hq+2Hkv)*d]) and k by the rotary embedding when
 * rope != 0 (pairs i, i+d/2; angle tok_pos * inv_freq[i], inv_freq fp32 [d/2]); write the
 * new k and v rows into kv (and into mirror, a second copy of the slice, if non-NULL).
 * k and v are rounded to kv_value_dtype and stored in containers of type dtype: a
 * bfloat16-valued cache can live in float16 containers (pairs f16/f16, f16/bf16,
 * bf16/bf16). */
int sn_k_rope_append(int32_t dtype, int32_t kv_value_dtype, void* qkv16, const int32_t* tok_seq, const int32_t* tok_pos,
                     const int32_t* kv_off, const int32_t* cap, void* kv, void* mirror,
                     const float* inv_freq, int32_t T, int32_t Hq, int32_t Hkv, int32_t d,
                     int32_t rope, void* stream);

/* One query per sequence (row b of qkv16) over keys 0..len_before[b] (the new row was
 * appended first).  out16 [B][Hq*d].  splits S >= 1 key ranges; part: fp32 scratch
 * [B][Hq][S][d+2] (may be NULL when S == 1).  S == 0: the library's own choice for
 * max_len = max_b(len_before[b]) + 1, which must then be given.  packed_out != 0: out16
 * is written row-tile packed (K = Hq*d).  Performance note on the cap array: capacities for
 * which cap[b] * d * 4 bytes is a multiple of 2^19 + 2^12 (1032 rows at d = 128) put every
 * (sequence, KV head) region on the same memory channels at the same time and run at less than
 * half speed; sn_kv_reset lays such sequences out with 8 rows more. */
int sn_k_attn_decode(int32_t dtype, const void* qkv16, const void* kv, const int32_t* len_before,
                     const int32_t* kv_off, const int32_t* cap, void* out16, float* part, int32_t B,
                     int32_t Hq, int32_t Hkv, int32_t d, int32_t S, int32_t max_len,
                     int32_t packed_out, void* stream);

/* sn_k_attn_decode for callers that cannot allocate device memory -- code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc: the partial results of the S key ranges go to a
 * buffer of SN_K_STATIC_SCRATCH_BYTES that is part of the library's code object, so there is no `part`
 * argument and the call allocates nothing (no hipMalloc / hipFree, no allocating library routine).  Inputs
 * and outputs are the caller's, as in sn_k_attn_decode, and the result is the same bit for bit.
 * Limit: B*Hq*S*(d+2)*4 bytes <= SN_K_STATIC_SCRATCH_BYTES when S > 1 (S == 0: the library's choice for
 * max_len, as in sn_k_attn_decode); beyond it SN_E_INVAL, with the sizes in sn_last_error(NULL).
 * Every call on one GPU uses that GPU's single buffer: calls that overlap on one GPU (different streams
 * or threads) race; calls on one stream are ordered.  Nothing in it needs clearing between calls (every
 * partial is written before it is read).  Each GPU the library has run on keeps its buffer until the
 * process ends; its address is looked up at sn_init or at the first call on that GPU. */
#define SN_K_STATIC_SCRATCH_BYTES (16u << 20)
int sn_k_attn_decode_static(int32_t dtype, const void* qkv16, const void* kv, const int32_t* len_before,
                            const int32_t* kv_off, const int32_t* cap, void* out16, int32_t B, int32_t Hq,
                            int32_t Hkv, int32_t d, int32_t S, int32_t max_len, int32_t packed_out,
                            void* stream);

/* The decode step's rotation, KV append and attention in one kernel (what sn_step runs
 * when decoding; steps a6 + a7 of a layer).  Row b of qkv16 is the QKV projection's
 * output as is: q and k not yet rotated, nothing appended.  The kernel rotates q and k at
 * position len_before[b] (rope != 0; inv_freq [d/2] device fp32), rounds them to the 16-bit
 * type, stores k and v as row len_before[b] of the sequence's slice in `kv` (device,
 * read and written) and in `mirror` (a second slice of identical layout, e.g. mapped
 * pinned host memory; may be NULL), and attends over keys 0..len_before[b].  qkv16 is not
 * modified.  Other arguments as sn_k_attn_decode.  Needs cap[b] > len_before[b] (not checked:
 * the arrays are device memory). */
int sn_k_attn_decode_append(int32_t dtype, const void* qkv16, void* kv, void* mirror, const float* inv_freq,
                            int32_t rope, const int32_t* len_before, const int32_t* kv_off,
                            const int32_t* cap, void* out16, float* part, int32_t B, int32_t Hq,
                            int32_t Hkv, int32_t d, int32_t S, int32_t max_len, int32_t packed_out,
                            void* stream);

/* sn_k_attn_decode_append with the step's q, k and v given as split-K partial planes of the QKV
 * projection (what sn_step runs at 9..128 rows, where that projection is split over K like the residual
 * projections; steps a5-a7): qkv_part [splits][plane_rows][(Hq + 2 Hkv) d] device fp32, 1 <= splits <= 8,
 * plane_rows >= B, the projection's bias already in plane 0 (sn_k_gemm_splitk writes exactly this).  The
 * kernel adds the planes in ascending order, rounds the sum to the 16-bit type -- the value the unsplit
 * projection stores -- and proceeds as sn_k_attn_decode_append.  qkv_part is not modified. */
int sn_k_attn_decode_append_planes(int32_t dtype, const float* qkv_part, int32_t splits, int32_t plane_rows,
                                   void* kv, void* mirror, const float* inv_freq, int32_t rope,
                                   const int32_t* len_before, const int32_t* kv_off, const int32_t* cap,
                                   void* out16, float* part, int32_t B, int32_t Hq, int32_t Hkv, int32_t d,
                                   int32_t S, int32_t max_len, int32_t packed_out, void* stream);

#define SN_K_PREFILL_QTILE 128
/* Causal attention of each sequence's n_new tokens over len_before+n_new keys.
 * out16 [T][Hq*d]; packed_out != 0: written row-tile packed (16*ceil(T/16) rows; needs Hq*d % 32 == 0). */
int sn_k_attn_prefill(int32_t dtype, const void* qkv16, const void* kv, const int32_t* len_before,
                      const int32_t* n_new, const int32_t* tok_start, const int32_t* kv_off,
                      const int32_t* cap, const int32_t* tile_seq, const int32_t* tile_q0,
                      void* out16, int32_t n_qtiles, int32_t Hq, int32_t Hkv, int32_t d, int32_t packed_out,
                      void* stream);

/* 16-bit <-> fp32 residual stream conversions at the boundary of an iteration. */
int sn_k_cast_in(int32_t dtype, const void* in16, void* x32, uint64_t n, void* stream);
int sn_k_cast_out(int32_t dtype, const void* x32, void* out16, uint64_t n, void* stream);

/* Plain device-to-device copy of `bytes` (multiple of 16): a kernel whose HBM traffic is
 * known exactly (bytes read + bytes written), used to calibrate hardware counters. */
int sn_k_copy(const void* src, void* dst, uint64_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SN_KERNELS_H_ */
