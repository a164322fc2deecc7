/*
 * sn.h -- C ABI of the SELECT-N offloaded serving iteration for one MI355X (gfx950).
 *
 * The library runs a decoder-only model layer by layer (paper Sec. 2.1).  With an
 * offloading interval N, the last layer of every group of N layers keeps its state
 * (weights and KV-cache slice) in pinned host memory; its load into one of two
 * device staging slots is issued on a copy stream when compute reaches the first
 * layer of the group, and a fence precedes the offloaded layer (Sec. 4.3, Fig. 7).
 * A profiler measures each layer's compute time and transfer time (Sec. 4.4) and a
 * picker returns the smallest interval whose iteration time meets a latency SLO,
 * bounded above by the GPU memory budget (Sec. 4.3 last paragraph, Sec. 4.5).
 *
 * Conventions
 *   - every function returns SN_OK (0) or a negative SN_E_* code; nothing aborts or
 *     throws across this boundary.  sn_last_error() gives a message for the last
 *     failing call on that context (or on the calling thread when ctx is NULL).
 *   - "host" / "device" is stated for every pointer.  Device pointers are plain HIP
 *     device addresses on the current device; the compute stream is a hipStream_t
 *     passed as void* (NULL = the default stream).
 *   - layers are numbered from 0; the paper numbers them from 1.
 *   - one context is used from one host thread at a time.
 */
#ifndef SN_H_
#define SN_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sn_ctx sn_ctx;

enum { SN_F16 = 0, SN_BF16 = 1 };
enum { SN_ACT_GELU = 0, SN_ACT_SWIGLU = 1 };
enum { SN_NORM_LN = 0, SN_NORM_RMS = 1 };

enum {
  SN_OK = 0,
  SN_E_INVAL = -1,      /* bad argument (null, out of range, unsupported shape)            */
  SN_E_STATE = -2,      /* call order: e.g. sn_step before sn_place, profile not taken      */
  SN_E_BUDGET = -3,     /* resident bytes for this interval exceed the HBM budget           */
  SN_E_INFEASIBLE = -4, /* no interval meets the SLO within capacity: reject (Sec. 4.2/4.5) */
  SN_E_NOMEM = -5,      /* host or device allocation failed                                 */
  SN_E_HIP = -6         /* a HIP runtime call failed                                        */
};

/* Decoder layer shape (Sec. 2.1: all layers share one structure). */
typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn;
  int32_t act;        /* SN_ACT_*  : GELU MLP (up, down) or SwiGLU MLP (gate, up, down)   */
  int32_t norm;       /* SN_NORM_* : LayerNorm (gain, shift) or RMSNorm (gain)            */
  int32_t rope;       /* 1: rotary embedding on q,k (pairs i, i+head_dim/2)               */
  int32_t has_bias;   /* 1: every projection has a bias vector                            */
  int32_t dtype;      /* SN_F16 / SN_BF16: type of the caller's weights and hidden in/out.  The library
                         computes in float16 either way (bfloat16 weights are stored as the equal
                         float16 value; the KV cache and all hand-offs are float16)          */
  float norm_eps, rope_theta;
  int32_t max_batch;  /* most sequences in one iteration                                   */
  int32_t max_seq;    /* sum of per-sequence KV capacities may not exceed max_batch*max_seq*/
  int32_t max_tokens; /* most tokens in one iteration (0: max_batch*max_seq)               */
} sn_model_shape;

/* One iteration's input (Sec. 2.1: prefill processes the whole prompt, decoding one
 * token per sequence).  Tokens of sequence b are rows tok_start(b)..+n_new[b] of
 * hidden_in, sequences in order. */
typedef struct {
  int32_t batch;
  int32_t is_prefill;       /* 0: decode (every n_new[b] == 1, batch <= 128); 1: prefill / chunk */
  const int32_t* n_new;     /* host, [batch]                                                */
  const void* hidden_in;    /* device, [sum n_new, hidden], shape.dtype                     */
} sn_batch;

/* KV bookkeeping.  Storage belongs to the context; the caller owns this small struct. */
typedef struct {
  int32_t* len;             /* host, [batch]: tokens cached per sequence; advanced by sn_step */
} sn_kv;

/* Timings of the most recent sn_step (valid once the compute stream has been
 * synchronised).  All times in nanoseconds from HIP events. */
typedef struct {
  int64_t iter_ns;          /* whole iteration on the compute stream                        */
  int64_t stall_ns;         /* time compute waited at fences (sum over offloaded layers)    */
  int64_t h2d_ns, h2d_bytes;/* summed duration and bytes of this iteration's prefetches     */
  int64_t d2h_ns, d2h_bytes;/* write-back copies (prefill); decode writes rows through      */
  double hidden_fraction;   /* 1 - stall_ns / h2d_ns (1 when nothing is offloaded)          */
  int32_t interval;         /* N in effect (n_layers+1: nothing offloaded)                  */
  int32_t n_offloaded;
  uint64_t resident_bytes;  /* device bytes held for this placement                         */
  int64_t kernel_ns[8];     /* per kernel class, summed over layers, when kernel timing on  */
  int32_t kernel_calls[8];
  int32_t n_preissued;      /* of this iteration's loads, how many had been issued during the
                               previous iteration (SN_SCHED_CONTINUOUS)                      */
  int32_t nonfinite;        /* 1: some hidden state of this iteration's output is inf or NaN.
                               All arithmetic runs in float16 with fp32 accumulation (bfloat16
                               models too: their weights are converted at load), activations
                               pass between kernels in float16, so a value beyond +-65504
                               overflows there; it then reaches the fp32 residual stream and
                               this flag.  0 for a healthy model.                            */
} sn_step_stats;

/* Kernel classes for sn_step_stats.kernel_ns / sn_set_timing(level 2). */
enum { SN_K_NORM = 0, SN_K_QKV = 1, SN_K_ROPE_APPEND = 2, SN_K_ATTN = 3, SN_K_OPROJ = 4,
       SN_K_FFN_UP = 5, SN_K_FFN_DOWN = 6, SN_K_OTHER = 7 };

/* --- life cycle ---------------------------------------------------------------- */

/* Create a context for a model of this shape under an HBM budget (Sec. 4.5: the
 * maximum interval follows from the GPU's capacity).  hbm_budget_bytes == 0: no cap.
 * Allocates the pinned host master for all layers' weights and the device workspace.
 * hip_compute_stream: caller-owned hipStream_t on which sn_step enqueues kernels.
 * The first call on a device in a process also runs a burst of small copies on
 * temporary streams (64 MB of pinned and of device memory for ~40 ms, released
 * before it returns), so that the runtime's one-off copy-queue set-ups, each of
 * which holds the calling thread for milliseconds, do not fall into an iteration. */
int sn_init(sn_ctx** out, const sn_model_shape* shape, uint64_t hbm_budget_bytes,
            void* hip_compute_stream);
void sn_destroy(sn_ctx* ctx);
const char* sn_last_error(const sn_ctx* ctx);
int32_t sn_layers(const sn_ctx* ctx);        /* the model's layer count; 0 for a null context */

/* --- weights -------------------------------------------------------------------
 * Caller-side layer blob: the tensors below in this order, 16-bit (shape.dtype),
 * matrices [out_features, in_features] row-major, each tensor starting on a 256-byte
 * boundary; tensors that the shape does not have are absent:
 *   wqkv [(Hq+2Hkv)*d, hidden] (q heads, then k heads, then v heads), bqkv,
 *   wo [hidden, Hq*d], bo, wg [ffn, hidden] (SwiGLU gate), bg, wu [ffn, hidden], bu,
 *   wd [hidden, ffn], bd, n1g [hidden], n1b (LayerNorm only), n2g, n2b.
 * sn_layer_blob_bytes gives the total size.  sn_set_layer_weights copies (and
 * re-tiles for the matrix cores); host_blob is a host pointer and may be freed
 * afterwards.  It may be called before or after sn_place.  Where the copy goes: a
 * layer that is host-resident, or that has not been placed yet, gets a pinned host
 * master; a layer that is GPU resident is written to its device copy (and to its
 * master, if it has one).  Masters are created when a layer first needs one and
 * then kept; when pinned memory runs out, masters of GPU-resident layers are given
 * up (a later sn_place copies such a layer back from the device).  For a model
 * whose weights exceed the host's pinned memory, call sn_place first.
 * SN_E_NOMEM if a master cannot be allocated even so. */
uint64_t sn_layer_blob_bytes(const sn_model_shape* shape);
int sn_set_layer_weights(sn_ctx* ctx, int32_t layer, const void* host_blob, uint64_t bytes);

/* --- placement (Sec. 4.3) ------------------------------------------------------
 * Apply offloading interval N: layer l is host resident iff (l+1) % N == 0.
 * N == 0 or N > n_layers: everything GPU resident.  Synchronous; moves weights and
 * live KV between host and device as needed; its cost is not part of an iteration.
 * Fails with SN_E_BUDGET when sn_resident_bytes(N) exceeds the budget, unless
 * enforcement was switched off with sn_set_budget_enforce(ctx, 0). */
int sn_place(sn_ctx* ctx, int32_t N);
int sn_set_budget_enforce(sn_ctx* ctx, int32_t on);
/* When the load of an offloaded layer is issued.
 *   SN_SCHED_PAPER (default): when compute reaches the first layer of the offloaded layer's own
 *     group (Sec. 4.3, Fig. 7; the previous layer when N = 1).
 *   SN_SCHED_EAGER: one group earlier -- as early as the two staging slots allow: the slot of
 *     the k-th offloaded layer is free once the (k-2)-th has been computed, so its load is
 *     issued at the layer after that one (at the start of the iteration for the first two).
 *     The copy stream then runs back to back, the regime the analyzer's closed form (Sec. 4.4)
 *     describes; the iteration is never longer than with SN_SCHED_PAPER, the output identical.
 *   SN_SCHED_CONTINUOUS: as SN_SCHED_EAGER within an iteration, and the loads do not stop at the
 *     iteration boundary (the paper is silent on the boundary; Sec. 4.4's closed form counts the
 *     transfers that fit into one iteration, which presumes this).  With K layers on the host,
 *     a decode iteration issues, as soon as its k-th host-resident layer has been computed, the
 *     load that the next iteration needs (number k + min(2, K) - K, if positive), weights and
 *     the whole KV slice, into the staging slot that has just become free.  The next sn_step
 *     finds those loads issued, whatever its kind; sn_place, sn_kv_reset, sn_set_schedule,
 *     sn_set_layer_weights and sn_profile_layers wait for them and discard them.  Prefill
 *     iterations run as SN_SCHED_EAGER (what follows a prefill needs the KV it writes back).
 *     sn_timeline_sched reports the steady state: the longer of the last two of 16 back-to-back
 *     iterations; the first iteration after a placement starts cold, as SN_SCHED_EAGER.
 * Takes effect at once (also for the placement in force); sn_pick_interval and the timeline it
 * uses follow the context's schedule. */
enum { SN_SCHED_PAPER = 0, SN_SCHED_EAGER = 1, SN_SCHED_CONTINUOUS = 2 };
int sn_set_schedule(sn_ctx* ctx, int32_t schedule);
/* Which part of a host-resident layer's state is kept on the host (the paper speaks of "LLM state",
 * Sec. 1, 2.3; both parts is the default).
 *   SN_OFFLOAD_STATE:   weights and KV slice; a load moves both (weights only in a prefill from
 *                       empty caches), new KV rows return to the host.
 *   SN_OFFLOAD_WEIGHTS: the weights; the layer's KV slice stays on the GPU, loads move weights
 *                       only, nothing returns to the host.
 *   SN_OFFLOAD_KV:      the KV slice; the weights stay on the GPU, a load moves the cached K/V
 *                       (nothing in a prefill from empty caches), new rows return to the host.
 * The part left behind stays on the GPU and a staging slot holds only the part that travels,
 * which sn_resident_bytes, sn_max_interval and the budget check follow.  Under a placement in
 * force the layers' parts are moved at once (synchronously, like sn_place; SN_E_BUDGET and no
 * change if the new footprint exceeds the budget).  The output does not depend on it.  A profile
 * taken before the change is dropped (its transfer times were for the other part). */
enum { SN_OFFLOAD_STATE = 0, SN_OFFLOAD_WEIGHTS = 1, SN_OFFLOAD_KV = 2 };
int sn_set_offload_part(sn_ctx* ctx, int32_t what);
int32_t sn_offload_part(const sn_ctx* ctx);      /* -1 for a null context */
/* Device bytes interval N needs: resident layers' state + what host-resident layers leave on the
 * GPU + two staging slots (if any layer is offloaded) + workspace. */
uint64_t sn_resident_bytes(const sn_ctx* ctx, int32_t N);
/* Largest N whose footprint fits the budget; n_layers+1 = "no offloading fits"
 * (infinite maximum, Sec. 4.5); 0 = not even N = 1 fits. */
int32_t sn_max_interval(const sn_ctx* ctx);

/* "Max length" of Sec. 5.6 (batch size x (sequence + output length)): the largest number of
 * cached tokens for which interval N (0 or > L: nothing offloaded) fits budget_bytes, when a
 * layer's state is weight_bytes_per_layer + tokens * kv_bytes_per_token_per_layer, the GPU holds
 * one state per resident layer plus two staging slots if anything is offloaded, and fixed_bytes
 * of workspace.  0 if not even the weights fit (or if a token costs nothing).  Pure, host only. */
uint64_t sn_max_tokens(int32_t L, int32_t N, uint64_t weight_bytes_per_layer, uint64_t kv_bytes_per_token_per_layer,
                       uint64_t fixed_bytes, uint64_t budget_bytes);
/* The same for a given part kept on the host (SN_OFFLOAD_*), and the footprint itself for a KV
 * slice of kv_bytes_per_layer.  0 for an unknown part.  Pure, host only. */
uint64_t sn_max_tokens_part(int32_t L, int32_t N, uint64_t weight_bytes_per_layer, uint64_t kv_bytes_per_token_per_layer,
                            uint64_t fixed_bytes, uint64_t budget_bytes, int32_t what);
uint64_t sn_resident_bytes_part(int32_t L, int32_t N, uint64_t weight_bytes_per_layer, uint64_t kv_bytes_per_layer,
                                uint64_t fixed_bytes, int32_t what);

/* Pure helpers (host only, no GPU): the placement map and prefetch triggers for
 * (L, N).  offloaded[l] in {0,1}; trigger[l] = layer at whose start the load of
 * layer l is issued, or -1 for resident layers.  Both host arrays of length L. */
int sn_placement(int32_t L, int32_t N, uint8_t* offloaded, int32_t* trigger);
int sn_placement_sched(int32_t L, int32_t N, int32_t schedule, uint8_t* offloaded, int32_t* trigger);

/* --- KV cache ------------------------------------------------------------------
 * Start a new set of sequences: per-sequence capacities in tokens (host, [batch]);
 * sum must fit max_batch*max_seq.  All lengths become 0.  sn_step enforces the capacities
 * given here; the slice of a sequence may be laid out with 8 rows more where the context
 * has the room (a row count whose head-to-head stride, rows * head_dim * 4 bytes, is a
 * multiple of 2^19 + 2^12 bytes makes every attention workgroup hit the same memory channel
 * at the same time: less than half the bandwidth). */
int sn_kv_reset(sn_ctx* ctx, int32_t batch, const int32_t* capacity);

/* Shorten the cached sequences: len (host, [batch]) gives the new token counts, none larger than
 * the current one.  The rows beyond them are dropped (capacities and layout stay), so the next
 * iteration continues from there -- e.g. a rejected speculative continuation, or a benchmark
 * that runs the same decode steps under several placements after one prefill.  The caller
 * sets its own sn_kv.len to the same values.  Bookkeeping only: nothing is copied. */
int sn_kv_truncate(sn_ctx* ctx, int32_t batch, const int32_t* len);

/* --- one serving iteration (Sec. 4.3, Fig. 7) ----------------------------------
 * Enqueues the whole layer loop and returns without waiting for the GPU.
 * hidden_out: device, [sum n_new, hidden], shape.dtype: hidden states after the last
 * layer.  kv->len[b] must equal the context's own count and is advanced by n_new[b].
 * Results are valid after the caller synchronises the compute stream. */
int sn_step(sn_ctx* ctx, const sn_batch* batch, sn_kv* kv, void* hidden_out);

/* The hidden states of the last sn_step before their final rounding to shape.dtype:
 * the fp32 residual stream, [sum n_new, hidden].  dst: device, dst_bytes its size.
 * Enqueued on the compute stream; hidden_out of that step is exactly this tensor
 * rounded to nearest-even. */
int sn_read_hidden_f32(sn_ctx* ctx, void* dst, uint64_t dst_bytes);

/* timing level: 0 iteration + copies only, 1 also per layer, 2 also per kernel class */
int sn_set_timing(sn_ctx* ctx, int32_t level);
/* At level 2, bracket only launches of one kernel class (SN_K_*) with events, so that
 * measuring the dominant kernel perturbs the iteration as little as possible; -1: all. */
int sn_set_kernel_timing_class(sn_ctx* ctx, int32_t kernel_class);
/* Times one decode-phase projection kernel class (SN_K_QKV, SN_K_OPROJ, SN_K_FFN_UP,
 * SN_K_FFN_DOWN) on its own: launches it once per GPU-resident layer on that layer's
 * weights, `reps` rounds back to back on the compute stream for `batch` token rows,
 * bracketed by one pair of HIP events.  The workspace activations are used as they
 * are and are overwritten; call it between requests.  *total_ns / *launches is the
 * average launch duration (launch gaps included). */
int sn_time_kernel_class(sn_ctx* ctx, int32_t kernel_class, int32_t batch, int32_t reps,
                         int64_t* total_ns, int32_t* launches);
/* Waits for the last sn_step's kernels and write-backs (not for loads already issued for the
 * next iteration under SN_SCHED_CONTINUOUS), then fills *out for that step. */
int sn_get_stats(sn_ctx* ctx, sn_step_stats* out);
/* Per-layer figures of the last sn_step (timing level >= 1): host arrays [n_layers];
 * stall_ns[l] is 0 for resident layers.  Any pointer may be NULL. */
int sn_get_layer_times(sn_ctx* ctx, int64_t* compute_ns, int64_t* stall_ns, int64_t* h2d_ns);

/* Test switches for the ordering that Sec. 4.3 / Fig. 7 requires between the compute stream and
 * the copy streams.  They change when things happen, never what is computed: with any
 * combination the output must be bit-identical to a run without them.  Every added kernel ends
 * by itself (the delays are bounded waits).
 *   SN_DEBUG_POISON_SLOT:   before each load, once its staging slot has been released, a fill
 *                           kernel on the copy stream overwrites the bytes the load will bring
 *                           with 16-bit NaN patterns: whoever still reads the slot's previous
 *                           layer, or reads the slot before the load has landed, yields NaN.
 *   SN_DEBUG_DELAY_H2D:     the copy stream waits delay_us before each load (after the poison):
 *                           compute reaches the host-resident layer first and must stall at the
 *                           synchronisation point "S"; stall_ns grows by about the delay.
 *   SN_DEBUG_DELAY_COMPUTE: the compute stream waits delay_us at the start of every layer, after
 *                           the loads triggered there have been handed over: the copy stream gets
 *                           ahead, so a kernel of that layer that still read a slot released by the
 *                           previous layer would find the poison or the next layer's weights.
 *   SN_DEBUG_DELAY_D2H:     the write-back stream waits delay_us before each prefill write-back of
 *                           a KV slice: the next iteration's load of that slice, its rows written
 *                           through while decoding, and the reuse of the staging slot all have to
 *                           wait for the write-back.
 * delay_us: 0..20000.  Synchronises all streams; flags == 0 switches everything off. */
enum { SN_DEBUG_POISON_SLOT = 1, SN_DEBUG_DELAY_H2D = 2, SN_DEBUG_DELAY_COMPUTE = 4, SN_DEBUG_DELAY_D2H = 8 };
int sn_set_debug(sn_ctx* ctx, int32_t flags, int32_t delay_us);

/* --- profiler and picker (Sec. 4.4) --------------------------------------------
 * Runs `reps` iterations of the given kind (prefill of `seq` tokens per sequence, or
 * one decode step on `seq` cached tokens) on generated inputs under the current
 * placement and reports per layer the median compute time tc_ns[l] (fence waits
 * excluded) and the time tx_ns[l] of a host-to-device transfer of that layer's state
 * (the part of it that sn_set_offload_part keeps on the host: weights; plus its KV prefix for
 * decode), taken while the compute stream runs such iterations -- the condition under which
 * prefetches run.  Host arrays [n_layers]; either
 * may be NULL.  Discards any live KV contents (lengths return to 0). */
int sn_profile_layers(sn_ctx* ctx, int32_t is_prefill, int32_t batch, int32_t seq, int32_t reps,
                      int64_t* tc_ns, int64_t* tx_ns);

/* Iteration time (ns) of the Fig. 7 schedule for interval N given per-layer times;
 * stall_total_ns may be NULL.  Pure, host only. */
int sn_timeline(int32_t L, const int64_t* tc_ns, const int64_t* tx_ns, int32_t N,
                int64_t* iter_ns, int64_t* stall_total_ns);
/* Smallest N in 1..L whose timeline meets slo_ns; L+1 if only the un-offloaded
 * iteration does; then N must not exceed N_max (Sec. 4.5), else SN_E_INFEASIBLE.
 * Pure, host only. */
int sn_pick_interval_from_times(int32_t L, const int64_t* tc_ns, const int64_t* tx_ns,
                                int64_t slo_ns, int32_t N_max, int32_t* N_out);
/* The two above for a given schedule (SN_SCHED_*); sn_timeline and
 * sn_pick_interval_from_times are the SN_SCHED_PAPER case. */
int sn_timeline_sched(int32_t L, const int64_t* tc_ns, const int64_t* tx_ns, int32_t N, int32_t schedule,
                      int64_t* iter_ns, int64_t* stall_total_ns);
int sn_pick_interval_from_times_sched(int32_t L, const int64_t* tc_ns, const int64_t* tx_ns, int64_t slo_ns,
                                      int32_t N_max, int32_t schedule, int32_t* N_out);
/* Same, using the last sn_profile_layers result, the context's budget and its schedule. */
int sn_pick_interval(sn_ctx* ctx, double slo_ms, int32_t* N_out);
/* Sec. 4.3 / 4.4 order intervals by the layers they offload (smaller interval, more host memory) and take the
 * smallest that meets the SLO.  Where L is not a multiple of N, several intervals offload the same
 * floor(L / N) layers -- the same host memory and the same GPU footprint -- and the paper does not choose
 * between them.  N_out = among the intervals N' >= N with floor(L / N') == floor(L / N), the one with the
 * shortest iteration under `schedule` (the smallest on a tie; N itself is a candidate, so the result meets every
 * latency and capacity bound N meets).  N = L + 1 is returned unchanged.  Pure, host only; host arrays [L];
 * SN_E_INVAL for N outside 1..L+1, a negative time or an unknown schedule. */
int sn_refine_interval_from_times(int32_t L, const int64_t* tc_ns, const int64_t* tx_ns, int32_t N, int32_t schedule,
                                  int32_t* N_out);
/* Same, using the last sn_profile_layers result and the context's schedule (what one calls on sn_pick_interval's
 * answer); SN_E_STATE before any profile. */
int sn_refine_interval(sn_ctx* ctx, int32_t N, int32_t* N_out);

/* The analyzer's closed form (Sec. 4.4) for uniform times, reported beside the pick:
 * L_offload = floor(slo / t_trans); interval = floor(L / (L_offload + 1)) + 1. */
int32_t sn_paper_rule(int32_t L, int64_t t_trans_ns, int64_t slo_ns);

#ifdef __cplusplus
}
#endif
#endif /* SN_H_ */
