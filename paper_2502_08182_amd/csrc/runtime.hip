// The runtime memory manager and the C ABI (include/sn.h).
//
// Paper Sec. 4.3 / Fig. 7: compute proceeds layer by layer on one stream; the state of
// each offloaded layer is loaded on a copy stream, the load being issued when compute
// reaches the first layer of the group, and a synchronisation point precedes the
// offloaded layer; afterwards its mutated state returns to the host.  Here:
//   * a host-resident layer keeps its (re-tiled) weights, its KV slice or both in pinned host
//     memory (sn_set_offload_part); what it leaves behind stays in device memory;
//   * two device staging slots for the part that travels, used alternately (the n-th load
//     issued goes to slot n mod 2);
//   * three schedules for issuing the loads (sn_set_schedule): the paper's, one group earlier,
//     and across the iteration boundary;
//   * an H2D stream (prefetch) and a D2H stream (write-back after prefill); during
//     decode the append kernel writes the new K/V rows through to the host slice, so
//     there is nothing left to copy back;
//   * HIP events as fences: trigger (compute -> copy), ready (copy -> compute),
//     slot-free (last reader of a slot -> next prefetch into it).
// Sec. 4.4: sn_profile_layers measures per-layer compute and transfer time; the picker
// (schedule.cpp) chooses the smallest interval whose timeline meets the SLO.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/sn.h"
#include "../../include/sn_kernels.h"
#include "kernels.h"
#include "layout.h"
#include "schedule.h"

using namespace sn;

namespace sn {
LaunchEvents& next_launch_events() {
  thread_local LaunchEvents le;
  return le;
}
}  // namespace sn

namespace {

thread_local std::string g_err;

constexpr int kMetaRing = 8;
constexpr int kKernelsPerLayer = 9;

struct LayerState {
  uint8_t* host_w = nullptr;    // pinned, tiled weights record: the host master.  Present while the layer is
                                // host-resident and kept afterwards as long as pinned memory lasts
  bool has_w = false;           // weights have been set (they live in host_w, in dev, or in both)
  uint8_t* host_kv = nullptr;   // pinned KV slice (present once the layer has been offloaded)
  uint8_t* host_kv_dev = nullptr;   // the same slice as the GPU addresses it (for write-through)
  uint8_t* dev_w = nullptr;     // device weights record, when the weights live on the GPU
  uint8_t* dev_kv = nullptr;    // device KV slice, when it lives on the GPU
  bool offloaded = false;       // some part of the layer's state lives on the host (it needs a load and a fence)
  bool w_host = false, kv_host = false;   // which part
  int slot = 0;                 // staging slot of the load in flight or last used (set when the load is issued)
  int trigger = -1;
  bool preissued = false;       // the load for the next iteration was issued during the previous one
  bool d2h_pending = false;     // a prefill's write-back of the KV slice (ev_d2h_end) has been enqueued and the
                                // compute stream has not waited for it yet
};

}  // namespace

// Scratch memory that belongs to the library's code object, for the entry point that may not allocate
// (sn_k_attn_decode_static).  Each GPU the library runs on holds its own copy until the process ends; in
// host code the array's name is only a handle, so its device address is looked up once per device, with
// that device current, and kept.
static __device__ __align__(256) unsigned char scratch[SN_K_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

// Device address of `scratch` on the current device (nullptr and a HIP error code on failure).
hipError_t static_scratch(void** out) {
  *out = nullptr;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}
}  // namespace

struct sn_ctx {
  sn_model_shape shape{};
  PackedLayout pl{};
  BlobLayout bl{};
  uint64_t budget = 0;
  bool enforce = true;
  hipStream_t compute = nullptr, h2d = nullptr, d2h = nullptr;
  int N = 0;                     // interval in effect (L+1: nothing offloaded)
  int sched = kSchedPaper;       // when prefetches are issued (sn_set_schedule)
  bool placed = false;
  int timing = 0;
  int timing_class = -1;          // kernel class whose launches are bracketed at level 2 (-1: all)
  int debug = 0;                  // SN_DEBUG_* switches (sn_set_debug)
  uint64_t debug_ticks = 0;       // length of a debug delay in wall-clock periods
  int debug_trips = 0;            // and the bound on its sleeps

  uint64_t w_bytes = 0, kv_bytes = 0, state_bytes = 0, ws_bytes = 0;
  int64_t max_tokens = 0;
  std::vector<LayerState> layers;
  int what = SN_OFFLOAD_STATE;   // which part of a host-resident layer's state is kept on the host
  uint8_t* slot_w[2] = {nullptr, nullptr};    // staging slots: the weights part and the KV part, present
  uint8_t* slot_kv[2] = {nullptr, nullptr};   // when that part travels
  uint8_t* stage_w = nullptr;    // pinned staging record for layers that have no host master

  // workspace (device)
  float* x32 = nullptr;
  uint16_t *u16 = nullptr, *qkv16 = nullptr, *attn16 = nullptr, *act16 = nullptr;
  float* part = nullptr;
  float* part32 = nullptr;       // split-K partial sums of the decode residual projections
  float* qkv_part32 = nullptr;   // split-K partial sums of the decode QKV projection (9..128 rows), see run_layer
  float* inv_freq = nullptr;
  int32_t* flag_dev = nullptr;   // set by the final cast of an iteration when a hidden state is not finite
  int32_t* meta_dev = nullptr;
  size_t meta_ints = 0;
  int32_t* meta_host[kMetaRing] = {};
  int32_t* meta_host_dev[kMetaRing] = {};   // the same pinned buffers as the GPU addresses them
  hipEvent_t ev_meta[kMetaRing] = {};
  bool meta_used[kMetaRing] = {};
  int meta_next = 0;

  // KV bookkeeping
  int batch = 0;
  std::vector<int32_t> cap, kv_off, len;   // cap: rows requested per sequence (the limit sn_step enforces)
  std::vector<int32_t> cap_rows;           // rows laid out per sequence: cap, or a few more (see sn_kv_reset)
  int64_t kv_used_tokens = 0;

  // events
  std::vector<hipEvent_t> ev_layer, ev_after_wait, ev_trig, ev_copy_start, ev_ready, ev_done, ev_d2h_start,
      ev_d2h_end;
  // ev_trig, ev_copy_start and ev_ready hold two sets of n_layers events, one per iteration parity:
  // a load issued ahead for the next iteration must not re-record what this iteration's statistics read
  hipEvent_t ev_slot_free[2] = {};
  bool slot_free_valid[2] = {false, false};
  int par = 0, last_par = 0;     // event set of the iteration being enqueued / of the last one enqueued
  uint32_t load_seq = 0;         // loads issued so far; a load goes to staging slot load_seq % 2
  hipEvent_t ev_iter_start = nullptr, ev_iter_end = nullptr;
  std::vector<hipEvent_t> kev;   // [L][kKernelsPerLayer][2], created on demand

  // what the last step did (for stats)
  bool last_valid = false;
  bool last_prefill = false;
  int last_tokens = 0;
  int last_timing = 0;
  int64_t last_h2d_bytes = 0, last_d2h_bytes = 0;
  int last_preissued = 0;        // loads of the last iteration that had been issued during the one before
  std::vector<uint8_t> last_kernel_class;   // [kKernelsPerLayer] class of each per-layer kernel slot

  // profile
  std::vector<int64_t> prof_tc, prof_tx;
  bool has_profile = false;

  std::string err;
};

namespace {

int fail(sn_ctx* c, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf;
  g_err = buf;
  return code;
}

#define SN_HIP(c, call)                                                                          \
  do {                                                                                           \
    hipError_t e_ = (call);                                                                      \
    if (e_ != hipSuccess)                                                                        \
      return fail((c), e_ == hipErrorOutOfMemory ? SN_E_NOMEM : SN_E_HIP, "%s: %s (%s:%d)", #call, \
                  hipGetErrorString(e_), __FILE__, __LINE__);                                    \
  } while (0)

uint64_t kv_token_bytes(const sn_model_shape& s) { return (uint64_t)2 * s.n_kv_heads * s.head_dim * 2; }

int64_t elapsed_ns(hipEvent_t a, hipEvent_t b) {
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, a, b) != hipSuccess) return -1;
  return (int64_t)std::llround((double)ms * 1.0e6);
}

int make_events(sn_ctx* c, std::vector<hipEvent_t>& v, int n, bool timing) {
  v.assign(n, nullptr);
  for (int i = 0; i < n; ++i)
    SN_HIP(c, hipEventCreateWithFlags(&v[i], timing ? hipEventDefault : hipEventDisableTiming));
  return SN_OK;
}

void free_events(std::vector<hipEvent_t>& v) {
  for (auto e : v)
    if (e) (void)hipEventDestroy(e);
  v.clear();
}

uint64_t fixed_bytes(const sn_ctx* c) { return c->ws_bytes; }

// What the last iteration's statistics need: its kernels and write-backs.  Every load it used has
// been waited for by the compute stream; the copy stream may already be busy with loads issued
// ahead for the next iteration, which must not be waited for here.
int sync_step(sn_ctx* c) {
  SN_HIP(c, hipStreamSynchronize(c->compute));
  SN_HIP(c, hipStreamSynchronize(c->d2h));
  return SN_OK;
}

int sync_all(sn_ctx* c) {
  SN_HIP(c, hipStreamSynchronize(c->compute));
  SN_HIP(c, hipStreamSynchronize(c->h2d));
  SN_HIP(c, hipStreamSynchronize(c->d2h));
  return SN_OK;
}

bool weights_travel(int what) { return what != SN_OFFLOAD_KV; }
bool kv_travels(int what) { return what != SN_OFFLOAD_WEIGHTS; }

// Debug delay on a stream (sn_set_debug): a bounded wait, enqueued like any kernel.
int debug_delay(sn_ctx* c, int flag, hipStream_t st) {
  if (!(c->debug & flag) || c->debug_ticks == 0) return SN_OK;
  SN_HIP(c, launch_delay(c->debug_ticks, c->debug_trips, st));
  return SN_OK;
}

// Loads issued ahead for an iteration that will not run as foreseen (placement, schedule, KV
// layout or weights are about to change): wait for the copy stream and forget them.  The staging
// slots then hold nothing anyone waits for.
int drop_preissued(sn_ctx* c) {
  bool any = false;
  for (auto& ls : c->layers) {
    any |= ls.preissued;
    ls.preissued = false;
  }
  if (any) SN_HIP(c, hipStreamSynchronize(c->h2d));
  return SN_OK;
}

// Hand the load of host-resident layer o to the copy stream: it starts once compute has reached
// this point (trigger) and the staging slot's previous user has been computed, fills the slot
// with the part of the layer's state that lives on the host, and signals ev_ready of event set `set`.
int issue_load(sn_ctx* c, int o, int set, bool with_kv, uint64_t kv_used, int64_t* bytes) {
  LayerState& os = c->layers[o];
  const int L = c->shape.n_layers;
  const int e = set * L + o;
  os.slot = (int)(c->load_seq++ & 1u);
  SN_HIP(c, hipEventRecord(c->ev_trig[e], c->compute));
  SN_HIP(c, hipStreamWaitEvent(c->h2d, c->ev_trig[e], 0));
  if (c->slot_free_valid[os.slot]) SN_HIP(c, hipStreamWaitEvent(c->h2d, c->ev_slot_free[os.slot], 0));
  // The host slice may still be receiving the KV a prefill produced (write-back on the D2H stream).  That copy
  // released the OTHER staging slot, so the slot-free event above does not order this load behind it.
  if (os.kv_host && with_kv && kv_used && os.d2h_pending) SN_HIP(c, hipStreamWaitEvent(c->h2d, c->ev_d2h_end[o], 0));
  const bool load_kv = os.kv_host && with_kv && kv_used;
  if (c->debug & SN_DEBUG_POISON_SLOT) {
    // the slot is free now: overwrite what the load is about to fill with 16-bit NaN patterns, so that anything
    // that still reads the slot's previous contents, or reads the slot before the load has landed, shows
    if (os.w_host) SN_HIP(c, launch_fill(c->slot_w[os.slot], c->w_bytes, 0x7e007e00u, c->h2d));
    if (load_kv) SN_HIP(c, launch_fill(c->slot_kv[os.slot], (kv_used + 15) / 16 * 16, 0x7e007e00u, c->h2d));
  }
  if (int rc = debug_delay(c, SN_DEBUG_DELAY_H2D, c->h2d)) return rc;
  SN_HIP(c, hipEventRecord(c->ev_copy_start[e], c->h2d));
  *bytes = 0;
  if (os.w_host) {
    SN_HIP(c, hipMemcpyAsync(c->slot_w[os.slot], os.host_w, c->w_bytes, hipMemcpyHostToDevice, c->h2d));
    *bytes += (int64_t)c->w_bytes;
  }
  if (load_kv) {
    SN_HIP(c, hipMemcpyAsync(c->slot_kv[os.slot], os.host_kv, kv_used, hipMemcpyHostToDevice, c->h2d));
    *bytes += (int64_t)kv_used;
  }
  SN_HIP(c, hipEventRecord(c->ev_ready[e], c->h2d));
  return SN_OK;
}

}  // namespace

// =================================================================================
// pure helpers
// =================================================================================
extern "C" int sn_placement(int32_t L, int32_t N, uint8_t* offloaded, int32_t* trigger) {
  if (L < 1 || !offloaded || !trigger) return fail(nullptr, SN_E_INVAL, "sn_placement: bad argument");
  for (int l = 0; l < L; ++l) {
    offloaded[l] = is_offloaded(L, N, l) ? 1 : 0;
    trigger[l] = offloaded[l] ? trigger_of(N, l) : -1;
  }
  return SN_OK;
}

static bool bad_sched(int32_t s) { return s != kSchedPaper && s != kSchedEager && s != kSchedContinuous; }

extern "C" int sn_placement_sched(int32_t L, int32_t N, int32_t schedule, uint8_t* offloaded, int32_t* trigger) {
  if (L < 1 || !offloaded || !trigger || bad_sched(schedule)) return fail(nullptr, SN_E_INVAL, "sn_placement_sched: bad argument");
  for (int l = 0; l < L; ++l) {
    offloaded[l] = is_offloaded(L, N, l) ? 1 : 0;
    trigger[l] = offloaded[l] ? trigger_of(N, l, schedule) : -1;
  }
  return SN_OK;
}

extern "C" int sn_timeline_sched(int32_t L, const int64_t* tc, const int64_t* tx, int32_t N, int32_t schedule,
                                 int64_t* iter_ns, int64_t* stall_total_ns) {
  if (L < 1 || !tc || !tx || !iter_ns || bad_sched(schedule)) return fail(nullptr, SN_E_INVAL, "sn_timeline_sched: bad argument");
  for (int l = 0; l < L; ++l)
    if (tc[l] < 0 || tx[l] < 0) return fail(nullptr, SN_E_INVAL, "sn_timeline_sched: negative time");
  *iter_ns = iteration_time(L, tc, tx, N, stall_total_ns, schedule);
  return SN_OK;
}

extern "C" int sn_pick_interval_from_times_sched(int32_t L, const int64_t* tc, const int64_t* tx, int64_t slo_ns,
                                                 int32_t N_max, int32_t schedule, int32_t* N_out) {
  if (L < 1 || !tc || !tx || !N_out || bad_sched(schedule))
    return fail(nullptr, SN_E_INVAL, "sn_pick_interval_from_times_sched: bad argument");
  for (int l = 0; l < L; ++l)
    if (tc[l] < 0 || tx[l] < 0) return fail(nullptr, SN_E_INVAL, "sn_pick_interval_from_times_sched: negative time");
  const int n = min_interval(L, tc, tx, slo_ns, schedule);
  if (n < 0) return fail(nullptr, SN_E_INFEASIBLE, "SLO %lld ns is below the un-offloaded iteration time", (long long)slo_ns);
  if (n > N_max)
    return fail(nullptr, SN_E_INFEASIBLE, "minimum interval %d exceeds the maximum %d allowed by GPU capacity", n, N_max);
  *N_out = n;
  return SN_OK;
}

extern "C" int sn_refine_interval_from_times(int32_t L, const int64_t* tc, const int64_t* tx, int32_t N, int32_t schedule,
                                             int32_t* N_out) {
  if (L < 1 || !tc || !tx || !N_out || N < 1 || N > L + 1 || bad_sched(schedule))
    return fail(nullptr, SN_E_INVAL, "sn_refine_interval_from_times: bad argument");
  for (int l = 0; l < L; ++l)
    if (tc[l] < 0 || tx[l] < 0) return fail(nullptr, SN_E_INVAL, "sn_refine_interval_from_times: negative time");
  *N_out = refine_interval(L, tc, tx, N, schedule);
  return SN_OK;
}

extern "C" int sn_timeline(int32_t L, const int64_t* tc, const int64_t* tx, int32_t N, int64_t* iter_ns,
                           int64_t* stall_total_ns) {
  if (L < 1 || !tc || !tx || !iter_ns) return fail(nullptr, SN_E_INVAL, "sn_timeline: bad argument");
  for (int l = 0; l < L; ++l)
    if (tc[l] < 0 || tx[l] < 0) return fail(nullptr, SN_E_INVAL, "sn_timeline: negative time");
  *iter_ns = iteration_time(L, tc, tx, N, stall_total_ns);
  return SN_OK;
}

extern "C" int sn_pick_interval_from_times(int32_t L, const int64_t* tc, const int64_t* tx, int64_t slo_ns,
                                           int32_t N_max, int32_t* N_out) {
  if (L < 1 || !tc || !tx || !N_out) return fail(nullptr, SN_E_INVAL, "sn_pick_interval_from_times: bad argument");
  for (int l = 0; l < L; ++l)
    if (tc[l] < 0 || tx[l] < 0) return fail(nullptr, SN_E_INVAL, "sn_pick_interval_from_times: negative time");
  const int n = min_interval(L, tc, tx, slo_ns);
  if (n < 0) return fail(nullptr, SN_E_INFEASIBLE, "SLO %lld ns is below the un-offloaded iteration time", (long long)slo_ns);
  if (n > N_max)
    return fail(nullptr, SN_E_INFEASIBLE, "minimum interval %d exceeds the maximum %d allowed by GPU capacity", n, N_max);
  *N_out = n;
  return SN_OK;
}

extern "C" uint64_t sn_max_tokens(int32_t L, int32_t N, uint64_t weight_bytes_per_layer, uint64_t kv_bytes_per_token_per_layer,
                                  uint64_t fixed_bytes, uint64_t budget_bytes) {
  if (L < 1 || N < 0) return 0;
  return max_tokens(L, N == 0 ? L + 1 : N, weight_bytes_per_layer, kv_bytes_per_token_per_layer, fixed_bytes, budget_bytes);
}

static bool bad_part(int32_t what) { return what != SN_OFFLOAD_STATE && what != SN_OFFLOAD_WEIGHTS && what != SN_OFFLOAD_KV; }

extern "C" uint64_t sn_max_tokens_part(int32_t L, int32_t N, uint64_t weight_bytes_per_layer, uint64_t kv_bytes_per_token_per_layer,
                                       uint64_t fixed_bytes, uint64_t budget_bytes, int32_t what) {
  if (L < 1 || N < 0 || bad_part(what)) return 0;
  return max_tokens(L, N == 0 ? L + 1 : N, weight_bytes_per_layer, kv_bytes_per_token_per_layer, fixed_bytes, budget_bytes, what);
}

extern "C" uint64_t sn_resident_bytes_part(int32_t L, int32_t N, uint64_t weight_bytes_per_layer, uint64_t kv_bytes_per_layer,
                                           uint64_t fixed_bytes, int32_t what) {
  if (L < 1 || N < 0 || bad_part(what)) return 0;
  return resident_bytes_of(L, N, weight_bytes_per_layer, kv_bytes_per_layer, fixed_bytes, what);
}

extern "C" int32_t sn_paper_rule(int32_t L, int64_t t_trans_ns, int64_t slo_ns) {
  return paper_rule(L, t_trans_ns, slo_ns);
}

extern "C" uint64_t sn_layer_blob_bytes(const sn_model_shape* shape) {
  if (!shape || check_shape(*shape)) return 0;
  return blob_layout(*shape).total;
}

extern "C" int32_t sn_layers(const sn_ctx* ctx) { return ctx ? ctx->shape.n_layers : 0; }

extern "C" const char* sn_last_error(const sn_ctx* ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

// =================================================================================
// life cycle
// =================================================================================
extern "C" void sn_destroy(sn_ctx* c) {
  if (!c) return;
  if (c->compute || c->h2d) {
    (void)hipStreamSynchronize(c->compute);
    if (c->h2d) (void)hipStreamSynchronize(c->h2d);
    if (c->d2h) (void)hipStreamSynchronize(c->d2h);
  }
  for (auto& ls : c->layers) {
    if (ls.host_w) (void)hipHostFree(ls.host_w);
    if (ls.host_kv) (void)hipHostFree(ls.host_kv);
    if (ls.dev_w) (void)hipFree(ls.dev_w);
    if (ls.dev_kv) (void)hipFree(ls.dev_kv);
  }
  for (auto& s : c->slot_w)
    if (s) (void)hipFree(s);
  for (auto& s : c->slot_kv)
    if (s) (void)hipFree(s);
  if (c->stage_w) (void)hipHostFree(c->stage_w);
  void* dev[] = {c->x32, c->u16, c->qkv16, c->attn16, c->act16, c->part, c->part32, c->qkv_part32, c->inv_freq, c->meta_dev, c->flag_dev};
  for (void* p : dev)
    if (p) (void)hipFree(p);
  for (int i = 0; i < kMetaRing; ++i) {
    if (c->meta_host[i]) (void)hipHostFree(c->meta_host[i]);
    if (c->ev_meta[i]) (void)hipEventDestroy(c->ev_meta[i]);
  }
  free_events(c->ev_layer);
  free_events(c->ev_after_wait);
  free_events(c->ev_trig);
  free_events(c->ev_copy_start);
  free_events(c->ev_ready);
  free_events(c->ev_done);
  free_events(c->ev_d2h_start);
  free_events(c->ev_d2h_end);
  free_events(c->kev);
  for (auto& e : c->ev_slot_free)
    if (e) (void)hipEventDestroy(e);
  if (c->ev_iter_start) (void)hipEventDestroy(c->ev_iter_start);
  if (c->ev_iter_end) (void)hipEventDestroy(c->ev_iter_end);
  if (c->h2d) (void)hipStreamDestroy(c->h2d);
  if (c->d2h) (void)hipStreamDestroy(c->d2h);
  delete c;
}

// The runtime sets up each of the device's copy queues the first time it picks that queue, which it does when the
// ones it knows are busy; the asynchronous copy call that hits such a set-up holds its thread for about 6 ms
// (measured: any copy size, any stream, a few times per process at unpredictable moments).  Inside an iteration that
// call is a prefetch, the thread is the one enqueueing the layers, and the compute stream runs dry behind it -- a
// single iteration of twice the usual length.  So the set-ups are provoked here, once per device and process:
// copies in flight on several streams at once, both directions.  Measured with 8 streams x 4 copies: the burst
// takes the stalls (two or three of them), and none was seen in the 1500 bursts of queued copies that followed,
// where without it one always was.
static int warm_copy_path(sn_ctx* c) {
  static std::mutex mu;
  static std::vector<int> done;
  std::lock_guard<std::mutex> guard(mu);
  int dev = 0;
  SN_HIP(c, hipGetDevice(&dev));
  if (std::find(done.begin(), done.end(), dev) != done.end()) return SN_OK;
  constexpr int kStreams = 8, kRounds = 4;
  constexpr size_t kBytes = (size_t)8 << 20;
  uint8_t *host = nullptr, *devbuf = nullptr;
  hipStream_t st[kStreams] = {};
  hipError_t e = hipHostMalloc((void**)&host, kStreams * kBytes, hipHostMallocDefault);
  if (e == hipSuccess) e = hipMalloc((void**)&devbuf, kStreams * kBytes);
  if (e == hipSuccess) std::memset(host, 0, kStreams * kBytes);
  for (int i = 0; i < kStreams && e == hipSuccess; ++i) e = hipStreamCreateWithFlags(&st[i], hipStreamNonBlocking);
  for (int dir = 0; dir < 2 && e == hipSuccess; ++dir) {
    for (int r = 0; r < kRounds; ++r)
      for (int i = 0; i < kStreams && e == hipSuccess; ++i)
        e = dir == 0 ? hipMemcpyAsync(devbuf + i * kBytes, host + i * kBytes, kBytes, hipMemcpyHostToDevice, st[i])
                     : hipMemcpyAsync(host + i * kBytes, devbuf + i * kBytes, kBytes, hipMemcpyDeviceToHost, st[i]);
    for (int i = 0; i < kStreams; ++i) {
      const hipError_t es = hipStreamSynchronize(st[i]);
      if (e == hipSuccess) e = es;
    }
  }
  for (int i = 0; i < kStreams; ++i)
    if (st[i]) (void)hipStreamDestroy(st[i]);
  if (devbuf) (void)hipFree(devbuf);
  if (host) (void)hipHostFree(host);
  if (e != hipSuccess)
    return fail(c, e == hipErrorOutOfMemory ? SN_E_NOMEM : SN_E_HIP, "copy path warm-up: %s", hipGetErrorString(e));
  done.push_back(dev);
  return SN_OK;
}

static int init_impl(sn_ctx* c, const sn_model_shape* shape, uint64_t budget, void* stream) {
  c->shape = *shape;
  const sn_model_shape& s = c->shape;
  c->budget = budget;
  c->compute = (hipStream_t)stream;
  c->pl = packed_layout(s);
  c->bl = blob_layout(s);
  c->w_bytes = c->pl.total;
  c->kv_bytes = align_up((uint64_t)s.max_batch * s.max_seq * kv_token_bytes(s));
  c->state_bytes = c->w_bytes + c->kv_bytes;
  c->max_tokens = s.max_tokens > 0 ? s.max_tokens : (int64_t)s.max_batch * s.max_seq;
  if (c->max_tokens < s.max_batch) c->max_tokens = s.max_batch;
  if (c->max_tokens > (int64_t)1 << 24) return fail(c, SN_E_INVAL, "max_tokens too large");
  const int L = s.n_layers;
  // activations between kernels are stored in 16-row tiles (decode always, prefill wherever the 256 x 256 projection kernel
  // runs): a tile that holds the last rows occupies its full 16-row footprint, so every row buffer keeps room for whole tiles
  const uint64_t T = (std::max<uint64_t>((uint64_t)c->max_tokens, (uint64_t)std::min(s.max_batch, kMaxDecodeRows)) + 15) / 16 * 16;
  const uint64_t qkv_ld = (uint64_t)c->pl.n_qkv, qd = (uint64_t)s.n_q_heads * s.head_dim;

  const uint64_t b_x32 = align_up(T * s.hidden * 4), b_u = align_up(T * s.hidden * 2);
  const uint64_t b_qkv = align_up(T * qkv_ld * 2), b_attn = align_up(T * qd * 2);
  const uint64_t b_act = align_up(T * (uint64_t)s.ffn * 2);
  const uint64_t b_part = align_up((uint64_t)s.max_batch * s.n_q_heads * 16 * (s.head_dim + 2) * 4);
  const uint64_t n_tiles_max = T / 64 + s.max_batch + 1;
  c->meta_ints = (size_t)(5 * (uint64_t)s.max_batch + 2 * T + 2 * n_tiles_max);
  const uint64_t b_meta = align_up(c->meta_ints * 4);
  const uint64_t b_freq = align_up((uint64_t)s.head_dim / 2 * 4);
  const uint64_t b_part32 = align_up((uint64_t)kMaxSplits * std::min(s.max_batch, kMaxDecodeRows) * s.hidden * 4);
  // a decode step of 9..128 rows may run its QKV projection split over K (gemm_qkv_splits)
  const uint64_t b_qkv_part = s.max_batch > 8 ? align_up((uint64_t)kMaxSplits * std::min(s.max_batch, kMaxDecodeRows) * qkv_ld * 4) : 0;
  c->ws_bytes = b_x32 + b_u + b_qkv + b_attn + b_act + b_part + b_part32 + b_qkv_part + b_meta + b_freq;

  SN_HIP(c, hipStreamCreateWithFlags(&c->h2d, hipStreamNonBlocking));
  SN_HIP(c, hipStreamCreateWithFlags(&c->d2h, hipStreamNonBlocking));
  if (int rc = warm_copy_path(c)) return rc;
  SN_HIP(c, hipMalloc(&c->x32, b_x32));
  SN_HIP(c, hipMalloc(&c->u16, b_u));
  SN_HIP(c, hipMalloc(&c->qkv16, b_qkv));
  SN_HIP(c, hipMalloc(&c->attn16, b_attn));
  SN_HIP(c, hipMalloc(&c->act16, b_act));
  SN_HIP(c, hipMalloc(&c->part, b_part));
  SN_HIP(c, hipMalloc(&c->part32, b_part32));
  if (b_qkv_part) SN_HIP(c, hipMalloc(&c->qkv_part32, b_qkv_part));
  SN_HIP(c, hipMalloc(&c->meta_dev, b_meta));
  SN_HIP(c, hipMalloc(&c->inv_freq, b_freq));
  SN_HIP(c, hipMalloc(&c->flag_dev, 256));
  SN_HIP(c, hipMemset(c->flag_dev, 0, 256));
  {
    std::vector<float> f(s.head_dim / 2);
    for (int i = 0; i < s.head_dim / 2; ++i)
      f[i] = (float)std::pow((double)s.rope_theta, -2.0 * i / (double)s.head_dim);
    SN_HIP(c, hipMemcpy(c->inv_freq, f.data(), f.size() * 4, hipMemcpyHostToDevice));
  }
  for (int i = 0; i < kMetaRing; ++i) {
    SN_HIP(c, hipHostMalloc((void**)&c->meta_host[i], b_meta, hipHostMallocDefault));
    SN_HIP(c, hipHostGetDevicePointer((void**)&c->meta_host_dev[i], c->meta_host[i], 0));
    SN_HIP(c, hipEventCreateWithFlags(&c->ev_meta[i], hipEventDisableTiming));
  }
  c->layers.resize(L);

  int rc;
  if ((rc = make_events(c, c->ev_layer, L + 1, true))) return rc;
  if ((rc = make_events(c, c->ev_after_wait, L, true))) return rc;
  if ((rc = make_events(c, c->ev_trig, 2 * L, false))) return rc;
  if ((rc = make_events(c, c->ev_copy_start, 2 * L, true))) return rc;
  if ((rc = make_events(c, c->ev_ready, 2 * L, true))) return rc;
  if ((rc = make_events(c, c->ev_done, L, false))) return rc;
  if ((rc = make_events(c, c->ev_d2h_start, L, true))) return rc;
  if ((rc = make_events(c, c->ev_d2h_end, L, true))) return rc;
  for (auto& e : c->ev_slot_free) SN_HIP(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
  SN_HIP(c, hipEventCreate(&c->ev_iter_start));
  SN_HIP(c, hipEventCreate(&c->ev_iter_end));
  c->prof_tc.assign(L, 0);
  c->prof_tx.assign(L, 0);
  return SN_OK;
}

extern "C" int sn_init(sn_ctx** out, const sn_model_shape* shape, uint64_t hbm_budget_bytes, void* stream) {
  if (!out || !shape) return fail(nullptr, SN_E_INVAL, "sn_init: null argument");
  *out = nullptr;
  if (const char* why = check_shape(*shape)) return fail(nullptr, SN_E_INVAL, "sn_init: %s", why);
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1)
    return fail(nullptr, SN_E_HIP, "sn_init: no HIP device available");
  {
    // set-up of the library's own scratch memory on this device, so that the entry point that must not
    // allocate finds it ready (it would otherwise do this on its first call)
    void* p = nullptr;
    const hipError_t e = static_scratch(&p);
    if (e != hipSuccess) return fail(nullptr, SN_E_HIP, "sn_init: address of the static scratch buffer: %s", hipGetErrorString(e));
  }
  sn_ctx* c = new sn_ctx();
  const int rc = init_impl(c, shape, hbm_budget_bytes, stream);
  if (rc != SN_OK) {
    g_err = c->err;
    sn_destroy(c);
    return rc;
  }
  *out = c;
  return SN_OK;
}

// =================================================================================
// weights, capacity accounting, placement
// =================================================================================
// A layer's host master is pinned memory.  Masters are created on demand (when a layer is
// host-resident, or when weights arrive before any placement) and then kept, so that a later
// re-placement needs no device-to-host copy; if pinned memory runs out, the masters of layers
// that currently live on the GPU are given up (their weights stay on the device) and the
// allocation is tried once more.
// N_keep: the placement that is in effect, or being established, when the call returns; only
// layers that are GPU-resident under it (and hold their weights on the device) may lose a master.
static int ensure_master(sn_ctx* c, int l, int N_keep) {
  LayerState& ls = c->layers[l];
  if (ls.host_w) return SN_OK;
  const int L = c->shape.n_layers;
  hipError_t e = hipHostMalloc((void**)&ls.host_w, c->w_bytes, hipHostMallocDefault);
  if (e == hipErrorOutOfMemory) {
    (void)hipGetLastError();
    ls.host_w = nullptr;
    for (int o = 0; o < L; ++o) {
      LayerState& os = c->layers[o];
      if (os.dev_w && os.host_w && (!is_offloaded(L, N_keep, o) || !weights_travel(c->what))) {
        (void)hipHostFree(os.host_w);
        os.host_w = nullptr;
      }
    }
    e = hipHostMalloc((void**)&ls.host_w, c->w_bytes, hipHostMallocDefault);
  }
  if (e != hipSuccess) {
    (void)hipGetLastError();
    ls.host_w = nullptr;
    return fail(c, e == hipErrorOutOfMemory ? SN_E_NOMEM : SN_E_HIP,
                "pinned host master of layer %d (%llu bytes): %s", l, (unsigned long long)c->w_bytes, hipGetErrorString(e));
  }
  return SN_OK;
}

static int ensure_stage(sn_ctx* c) {
  if (c->stage_w) return SN_OK;
  SN_HIP(c, hipHostMalloc((void**)&c->stage_w, c->w_bytes, hipHostMallocDefault));
  return SN_OK;
}

extern "C" int sn_set_layer_weights(sn_ctx* c, int32_t layer, const void* host_blob, uint64_t bytes) {
  if (!c) return fail(nullptr, SN_E_INVAL, "sn_set_layer_weights: null context");
  if (!host_blob || layer < 0 || layer >= c->shape.n_layers) return fail(c, SN_E_INVAL, "sn_set_layer_weights: bad layer or blob");
  if (bytes != c->bl.total)
    return fail(c, SN_E_INVAL, "sn_set_layer_weights: blob is %llu bytes, layout needs %llu", (unsigned long long)bytes,
                (unsigned long long)c->bl.total);
  int rc = sync_all(c);
  if (rc) return rc;
  for (auto& other : c->layers) other.preissued = false;     // a load issued ahead may carry the old weights
  LayerState& ls = c->layers[layer];
  // Destination of the tiled record: the layer's host master if it has one; a layer that lives
  // on the GPU and has no master is packed into the staging record and uploaded from there.
  uint8_t* dst = ls.host_w;
  if (!dst) {
    if (ls.dev_w) {
      if ((rc = ensure_stage(c))) return rc;
      dst = c->stage_w;
    } else {
      if ((rc = ensure_master(c, layer, c->placed ? c->N : c->shape.n_layers + 1))) return rc;
      dst = ls.host_w;
    }
  }
  // All arithmetic runs in float16 with fp32 accumulation.  bfloat16 weights are stored as
  // the equal float16 value (exact for 2^-17 <= |w| <= 65504): activations kept in
  // bfloat16 between kernels would lose 3 mantissa bits per hand-off, which at the
  // 13B/70B layer shapes is already ~3e-2 x RMS after a single layer.
  const uint64_t bad = pack_layer(c->shape, static_cast<const uint8_t*>(host_blob), dst);
  if (bad)
    return fail(c, SN_E_INVAL, "sn_set_layer_weights: %llu weights are not representable in float16 (|w| > 65504, inf or NaN)",
                (unsigned long long)bad);
  if (ls.dev_w) SN_HIP(c, hipMemcpy(ls.dev_w, dst, c->w_bytes, hipMemcpyHostToDevice));
  ls.has_w = true;
  return SN_OK;
}

extern "C" uint64_t sn_resident_bytes(const sn_ctx* c, int32_t N) {
  if (!c) return 0;
  return resident_bytes_of(c->shape.n_layers, N, c->w_bytes, c->kv_bytes, fixed_bytes(c), c->what);
}

extern "C" int32_t sn_max_interval(const sn_ctx* c) {
  if (!c) return 0;
  return max_interval_of(c->shape.n_layers, c->budget, c->w_bytes, c->kv_bytes, fixed_bytes(c), c->what);
}

extern "C" int sn_set_schedule(sn_ctx* c, int32_t schedule) {
  if (!c) return fail(nullptr, SN_E_INVAL, "null context");
  if (bad_sched(schedule)) return fail(c, SN_E_INVAL, "sn_set_schedule: unknown schedule %d", schedule);
  int rc = sync_all(c);
  if (rc) return rc;
  for (auto& ls : c->layers) ls.preissued = false;
  c->sched = schedule;
  if (c->placed)
    for (int l = 0; l < c->shape.n_layers; ++l) {
      LayerState& ls = c->layers[l];
      ls.trigger = ls.offloaded ? trigger_of(c->N, l, c->sched) : -1;
    }
  c->last_valid = false;
  return SN_OK;
}

extern "C" int sn_set_offload_part(sn_ctx* c, int32_t what) {
  if (!c) return fail(nullptr, SN_E_INVAL, "null context");
  if (bad_part(what)) return fail(c, SN_E_INVAL, "sn_set_offload_part: unknown part %d", what);
  if (what == c->what) return SN_OK;
  const int before = c->what;
  c->what = what;
  c->has_profile = false;          // transfer times were measured for the other part
  if (!c->placed) return SN_OK;
  const int rc = sn_place(c, c->N);  // moves what has to move; checks the budget first and changes nothing if it fails
  if (rc) c->what = before;
  return rc;
}

extern "C" int32_t sn_offload_part(const sn_ctx* c) { return c ? c->what : -1; }

extern "C" int sn_set_budget_enforce(sn_ctx* c, int32_t on) {
  if (!c) return fail(nullptr, SN_E_INVAL, "null context");
  c->enforce = on != 0;
  return SN_OK;
}

extern "C" int sn_place(sn_ctx* c, int32_t N) {
  if (!c) return fail(nullptr, SN_E_INVAL, "sn_place: null context");
  const int L = c->shape.n_layers;
  if (N < 0) return fail(c, SN_E_INVAL, "sn_place: negative interval");
  if (N == 0 || N > L) N = L + 1;
  const uint64_t need = sn_resident_bytes(c, N);
  if (c->enforce && c->budget && need > c->budget)
    return fail(c, SN_E_BUDGET, "interval %d needs %llu device bytes, budget is %llu", N, (unsigned long long)need,
                (unsigned long long)c->budget);
  int rc = sync_all(c);
  if (rc) return rc;
  for (auto& ls : c->layers) ls.preissued = false;      // loads issued ahead have landed; nobody will use them
  const uint64_t kv_used = (uint64_t)c->kv_used_tokens * kv_token_bytes(c->shape);

  // first release what leaves the GPU, then allocate what enters it
  auto w_goes_host = [&](int l) { return is_offloaded(L, N, l) && weights_travel(c->what); };
  auto kv_goes_host = [&](int l) { return is_offloaded(L, N, l) && kv_travels(c->what); };
  for (int l = 0; l < L; ++l) {
    LayerState& ls = c->layers[l];
    if (w_goes_host(l)) {
      if (!ls.host_w) {     // the weights move to (or start in) host memory: they need their master
        if ((rc = ensure_master(c, l, N))) return rc;
        if (ls.dev_w && ls.has_w) SN_HIP(c, hipMemcpy(ls.host_w, ls.dev_w, c->w_bytes, hipMemcpyDeviceToHost));
      }
      if (ls.dev_w) {
        SN_HIP(c, hipFree(ls.dev_w));
        ls.dev_w = nullptr;
      }
    }
    if (kv_goes_host(l)) {
      if (!ls.host_kv) {
        SN_HIP(c, hipHostMalloc((void**)&ls.host_kv, c->kv_bytes, hipHostMallocDefault));
        std::memset(ls.host_kv, 0, c->kv_bytes);
        SN_HIP(c, hipHostGetDevicePointer((void**)&ls.host_kv_dev, ls.host_kv, 0));
      }
      if (ls.dev_kv) {
        if (kv_used) SN_HIP(c, hipMemcpy(ls.host_kv, ls.dev_kv, kv_used, hipMemcpyDeviceToHost));
        SN_HIP(c, hipFree(ls.dev_kv));
        ls.dev_kv = nullptr;
      }
    }
  }
  const int K = offloaded_count(L, N);
  for (int i = 0; i < 2; ++i) {
    if ((K == 0 || !weights_travel(c->what)) && c->slot_w[i]) {
      SN_HIP(c, hipFree(c->slot_w[i]));
      c->slot_w[i] = nullptr;
    }
    if ((K == 0 || !kv_travels(c->what)) && c->slot_kv[i]) {
      SN_HIP(c, hipFree(c->slot_kv[i]));
      c->slot_kv[i] = nullptr;
    }
  }
  for (int l = 0; l < L; ++l) {
    LayerState& ls = c->layers[l];
    if (!w_goes_host(l) && !ls.dev_w) {
      SN_HIP(c, hipMalloc((void**)&ls.dev_w, c->w_bytes));
      if (ls.host_w) SN_HIP(c, hipMemcpy(ls.dev_w, ls.host_w, c->w_bytes, hipMemcpyHostToDevice));
    }
    if (!kv_goes_host(l) && !ls.dev_kv) {
      SN_HIP(c, hipMalloc((void**)&ls.dev_kv, c->kv_bytes));
      if (ls.host_kv && ls.kv_host && kv_used)      // the slice was live on the host until now
        SN_HIP(c, hipMemcpy(ls.dev_kv, ls.host_kv, kv_used, hipMemcpyHostToDevice));
      else
        SN_HIP(c, hipMemset(ls.dev_kv, 0, c->kv_bytes));
    }
  }
  if (K > 0)
    for (int i = 0; i < 2; ++i) {
      if (weights_travel(c->what) && !c->slot_w[i]) SN_HIP(c, hipMalloc((void**)&c->slot_w[i], c->w_bytes));
      if (kv_travels(c->what) && !c->slot_kv[i]) SN_HIP(c, hipMalloc((void**)&c->slot_kv[i], c->kv_bytes));
    }
  for (int l = 0; l < L; ++l) {
    LayerState& ls = c->layers[l];
    ls.offloaded = is_offloaded(L, N, l);
    ls.w_host = w_goes_host(l);
    ls.kv_host = kv_goes_host(l);
    ls.trigger = ls.offloaded ? trigger_of(N, l, c->sched) : -1;
    ls.slot = 0;
    ls.d2h_pending = false;          // every stream was waited for above
  }
  c->slot_free_valid[0] = c->slot_free_valid[1] = false;
  c->N = N;
  c->placed = true;
  c->last_valid = false;
  return SN_OK;
}

// =================================================================================
// KV bookkeeping
// =================================================================================
extern "C" int sn_kv_reset(sn_ctx* c, int32_t batch, const int32_t* capacity) {
  if (!c) return fail(nullptr, SN_E_INVAL, "sn_kv_reset: null context");
  if (batch < 1 || batch > c->shape.max_batch || !capacity) return fail(c, SN_E_INVAL, "sn_kv_reset: bad batch");
  int64_t tot = 0;
  for (int b = 0; b < batch; ++b) {
    if (capacity[b] < 1) return fail(c, SN_E_INVAL, "sn_kv_reset: capacity must be positive");
    tot += capacity[b];
  }
  if (tot > (int64_t)c->shape.max_batch * c->shape.max_seq)
    return fail(c, SN_E_INVAL, "sn_kv_reset: capacities sum to %lld tokens, context holds %lld", (long long)tot,
                (long long)c->shape.max_batch * c->shape.max_seq);
  int rc = drop_preissued(c);      // a load issued ahead carries the old layout's KV bytes
  if (rc) return rc;
  c->batch = batch;
  c->cap.assign(capacity, capacity + batch);
  c->cap_rows.assign(capacity, capacity + batch);
  c->kv_off.assign(batch, 0);
  c->len.assign(batch, 0);
  // The regions of consecutive KV heads lie 2 * rows * d * 2 bytes apart and the attention kernels stream all of
  // them at the same pace.  When that stride is a multiple of 2^19 + 2^12 bytes the memory channel hash sends the
  // k-th KiB of every region to the same channel (measured: 1032 rows at d = 128, 2.4 instead of 5.7 TB/s; 2064
  // rows 3.4 instead of 6.3), so such a sequence is laid out with 8 rows more -- where the context has the room.
  const int64_t limit = (int64_t)c->shape.max_batch * c->shape.max_seq;
  const int64_t row_bytes = (int64_t)c->shape.head_dim * 4;
  for (int b = 0; b < batch; ++b)
    if ((capacity[b] * row_bytes) % ((1 << 19) + (1 << 12)) == 0 && tot + 8 <= limit) {
      c->cap_rows[b] += 8;
      tot += 8;
    }
  int32_t off = 0;
  for (int b = 0; b < batch; ++b) {
    c->kv_off[b] = off;
    off += c->cap_rows[b];
  }
  c->kv_used_tokens = tot;
  return SN_OK;
}

extern "C" int sn_kv_truncate(sn_ctx* c, int32_t batch, const int32_t* len) {
  if (!c) return fail(nullptr, SN_E_INVAL, "sn_kv_truncate: null context");
  if (c->batch == 0) return fail(c, SN_E_STATE, "sn_kv_truncate before sn_kv_reset");
  if (batch != c->batch || !len) return fail(c, SN_E_INVAL, "sn_kv_truncate: batch %d, KV was reset for %d", batch, c->batch);
  for (int b = 0; b < batch; ++b)
    if (len[b] < 0 || len[b] > c->len[b])
      return fail(c, SN_E_INVAL, "sn_kv_truncate: sequence %d holds %d tokens, cannot become %d", b, c->len[b], len[b]);
  // Rows beyond the new lengths stay where they are and are never read again; a load issued ahead
  // carries the whole slice and stays valid.  Only the bookkeeping changes.
  for (int b = 0; b < batch; ++b) c->len[b] = len[b];
  return SN_OK;
}

extern "C" int sn_set_debug(sn_ctx* c, int32_t flags, int32_t delay_us) {
  if (!c) return fail(nullptr, SN_E_INVAL, "sn_set_debug: null context");
  const int known = SN_DEBUG_POISON_SLOT | SN_DEBUG_DELAY_H2D | SN_DEBUG_DELAY_COMPUTE | SN_DEBUG_DELAY_D2H;
  if (flags & ~known) return fail(c, SN_E_INVAL, "sn_set_debug: unknown flag in 0x%x", flags);
  if (delay_us < 0 || delay_us > 20000) return fail(c, SN_E_INVAL, "sn_set_debug: delay must be 0..20000 us");
  int dev = 0, khz = 0;
  SN_HIP(c, hipGetDevice(&dev));
  if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) {
    (void)hipGetLastError();
    khz = 100000;                     // the constant-rate counter of this GPU family runs at 100 MHz
  }
  int rc = sync_all(c);
  if (rc) return rc;
  c->debug = flags;
  c->debug_ticks = (uint64_t)delay_us * (uint64_t)khz / 1000u;
  c->debug_trips = delay_us;          // a sleep lasts a microsecond or more: the time test ends the wait first
  return SN_OK;
}

// =================================================================================
// one iteration
// =================================================================================
namespace {

struct KTimer {   // optional per-kernel event pairs (timing level 2)
  sn_ctx* c;
  int layer;
  int slot = 0;
  bool on;
  bool want(int cls) const { return on && (c->timing_class < 0 || c->timing_class == cls); }
  // The first kernel launched after begin() records its own start/stop timestamps.
  void begin(int cls) {
    if (want(cls)) {
      LaunchEvents& le = next_launch_events();
      le.start = c->kev[((size_t)layer * kKernelsPerLayer + slot) * 2];
      le.stop = c->kev[((size_t)layer * kKernelsPerLayer + slot) * 2 + 1];
    }
  }
  void end(int cls) {
    if (want(cls)) c->last_kernel_class[slot] = (uint8_t)cls;
    next_launch_events() = LaunchEvents{};
    ++slot;
  }
};

// `pending`: split-K partial sums of the previous residual projection that the next reader of
// the residual stream (a norm, or the final cast) folds in.
int run_layer(sn_ctx* c, int l, uint8_t* base, uint8_t* kv, uint8_t* mirror_kv, const StepIndex& ix, int T, int B,
              bool prefill, int n_qtiles, int S, Fold& pending) {
  const sn_model_shape& s = c->shape;
  const PackedLayout& p = c->pl;
  const int dt = SN_F16;   // compute and internal storage type (see sn_set_layer_weights)
  const int h = s.hidden, F = s.ffn, Hq = s.n_q_heads, Hkv = s.n_kv_heads, d = s.head_dim;
  const int qd = Hq * d;
  auto at = [&](uint64_t off) -> const void* { return off == kNone ? nullptr : base + off; };
  hipStream_t st = c->compute;
  const bool small = !prefill;   // decode path: T == B <= kMaxDecodeRows
  KTimer kt{c, l, 0, c->timing >= 2};
  // decode: activations between kernels are row-tile packed (inputs of the skinny GEMMs);
  // the QKV output stays row-major for the attention kernels
  const int pk = small ? 1 : 0;
  // prefill: a projection that runs on the 256 x 256 kernel reads its activations row-tile packed too (whole cache
  // lines per request), so whoever produces them writes that layout -- the norms, the attention kernel, and the FFN
  // up-projection when it is itself such a launch
  const bool pk_qkv = !small && gemm_tile_takes_packed(T, p.n_qkv, h), pk_up = !small && gemm_tile_takes_packed(T, p.n_up, h);
  const bool pk_o = !small && gemm_tile_takes_packed(T, h, qd), pk_down = pk_up && gemm_tile_takes_packed(T, h, F);
  auto gemm = [&](int epi, const void* W, const void* X, const void* bias, void* out, int N, int K, bool out_feeds_gemm,
                  bool x_packed, bool out_packed) {
    return small ? launch_gemm_skinny(dt, epi, W, X, bias, out, T, N, K, st, 1,
                                      kXPacked | (out_feeds_gemm ? kOutPacked : 0))
                 : launch_gemm_tile(dt, epi, W, X, bias, out, T, N, K, st, (x_packed ? kXPacked : 0) | (out_packed ? kOutPacked : 0));
  };
  // residual projection: decode writes split-K partials (folded in by the next norm / cast),
  // prefill adds into the residual stream in its epilogue
  auto resid_gemm = [&](const void* W, const void* X, const void* bias, int K, bool x_packed) -> hipError_t {
    if (!small) return launch_gemm_tile(dt, EPI_RESID32, W, X, bias, c->x32, T, h, K, st, x_packed ? kXPacked : 0);
    const int sp = gemm_skinny_splits(T, h, K);
    pending.part = c->part32;
    pending.nsplit = sp;
    pending.bias = nullptr;     // added by the GEMM into plane 0: the fold must not touch this layer's record
    return launch_gemm_skinny(dt, EPI_PART32, W, X, bias, c->part32, T, h, K, st, sp, kXPacked);
  };
  kt.begin(SN_K_NORM);
  SN_HIP(c, launch_norm_fold(dt, s.norm == SN_NORM_LN, c->x32, at(p.n1g), at(p.n1b), c->u16, T, h, s.norm_eps, pending, st, pk | (pk_qkv ? 1 : 0)));
  pending = Fold{};
  kt.end(SN_K_NORM);
  // decode, 9..128 rows: the QKV projection has too few output features to give every compute unit a
  // workgroup, so it is split over K like the residual projections; its fp32 planes are summed by the
  // attention kernel where it picks up the step's q, k and v
  const int qkv_splits = small && c->qkv_part32 ? gemm_qkv_splits(T, p.n_qkv, h) : 0;
  kt.begin(SN_K_QKV);
  if (qkv_splits)
    SN_HIP(c, launch_gemm_skinny(dt, EPI_PART32, at(p.wqkv), c->u16, at(p.bqkv), c->qkv_part32, T, p.n_qkv, h, st, qkv_splits, kXPacked));
  else
    SN_HIP(c, gemm(EPI_STORE16, at(p.wqkv), c->u16, at(p.bqkv), c->qkv16, p.n_qkv, h, false, pk_qkv, false));
  kt.end(SN_K_QKV);
  if (prefill) {
    kt.begin(SN_K_ROPE_APPEND);
    SN_HIP(c, launch_rope_append(dt, dt, c->qkv16, ix, kv, mirror_kv, c->inv_freq, T, Hq, Hkv, d, s.rope, st));
    kt.end(SN_K_ROPE_APPEND);
    kt.begin(SN_K_ATTN);
    SN_HIP(c, launch_attn_prefill(dt, c->qkv16, kv, ix, c->attn16, n_qtiles, Hq, Hkv, d, st, pk_o ? 1 : 0));
    kt.end(SN_K_ATTN);
  } else {
    // decode: rotation and KV append are done by the attention kernel itself
    AttnAppend ap{(uint16_t*)kv, (uint16_t*)mirror_kv, c->inv_freq, s.rope};
    if (qkv_splits) {
      ap.qkv_part = c->qkv_part32;
      ap.qkv_nsplit = qkv_splits;
      ap.qkv_rows = T;
    }
    kt.begin(SN_K_ATTN);
    SN_HIP(c, launch_attn_decode(dt, c->qkv16, kv, ix, c->attn16, c->part, B, Hq, Hkv, d, S, st, 1, &ap));
    kt.end(SN_K_ATTN);
  }
  kt.begin(SN_K_OPROJ);
  SN_HIP(c, resid_gemm(at(p.wo), c->attn16, at(p.bo), qd, pk_o));
  kt.end(SN_K_OPROJ);
  kt.begin(SN_K_NORM);
  SN_HIP(c, launch_norm_fold(dt, s.norm == SN_NORM_LN, c->x32, at(p.n2g), at(p.n2b), c->u16, T, h, s.norm_eps, pending, st, pk | (pk_up ? 1 : 0)));
  pending = Fold{};
  kt.end(SN_K_NORM);
  kt.begin(SN_K_FFN_UP);
  SN_HIP(c, gemm(s.act == SN_ACT_SWIGLU ? EPI_SWIGLU16 : EPI_GELU16, at(p.wup), c->u16, at(p.bup), c->act16, p.n_up, h, true, pk_up, pk_down));
  kt.end(SN_K_FFN_UP);
  kt.begin(SN_K_FFN_DOWN);
  SN_HIP(c, resid_gemm(at(p.wd), c->act16, at(p.bd), F, pk_down));
  kt.end(SN_K_FFN_DOWN);
  return SN_OK;
}

}  // namespace

extern "C" int sn_step(sn_ctx* c, const sn_batch* bt, sn_kv* kv, void* hidden_out) {
  if (!c) return fail(nullptr, SN_E_INVAL, "sn_step: null context");
  if (!c->placed) return fail(c, SN_E_STATE, "sn_step before sn_place");
  if (!bt || !kv || !kv->len || !bt->n_new || !bt->hidden_in || !hidden_out)
    return fail(c, SN_E_INVAL, "sn_step: null argument");
  if (c->batch == 0) return fail(c, SN_E_STATE, "sn_step before sn_kv_reset");
  if (bt->batch != c->batch) return fail(c, SN_E_INVAL, "sn_step: batch %d, KV was reset for %d", bt->batch, c->batch);
  const sn_model_shape& s = c->shape;
  const int B = c->batch, L = s.n_layers;
  const bool prefill = bt->is_prefill != 0;
  int64_t T64 = 0;
  bool any_cached = false;
  for (int b = 0; b < B; ++b) {
    if (kv->len[b] != c->len[b])
      return fail(c, SN_E_INVAL, "sn_step: kv.len[%d] = %d but the context holds %d", b, kv->len[b], c->len[b]);
    const int n = bt->n_new[b];
    if (n < 0 || (!prefill && n != 1)) return fail(c, SN_E_INVAL, "sn_step: n_new[%d] = %d", b, n);
    if (c->len[b] + n > c->cap[b])
      return fail(c, SN_E_INVAL, "sn_step: sequence %d would hold %d tokens, capacity %d", b, c->len[b] + n, c->cap[b]);
    any_cached |= c->len[b] > 0;
    T64 += n;
  }
  if (T64 == 0) return fail(c, SN_E_INVAL, "sn_step: no tokens");
  if (T64 > c->max_tokens) return fail(c, SN_E_INVAL, "sn_step: %lld tokens exceed max_tokens %lld", (long long)T64, (long long)c->max_tokens);
  if (!prefill && B > kMaxDecodeRows) return fail(c, SN_E_INVAL, "sn_step: decode batch above %d", kMaxDecodeRows);
  const int T = (int)T64;

  // ---- index arrays: host ring buffer -> device ----
  const int ring = c->meta_next;
  c->meta_next = (ring + 1) % kMetaRing;
  if (c->meta_used[ring]) SN_HIP(c, hipEventSynchronize(c->ev_meta[ring]));
  int32_t* mh = c->meta_host[ring];
  int32_t *m_len = mh, *m_new = mh + B, *m_start = mh + 2 * B, *m_off = mh + 3 * B, *m_cap = mh + 4 * B;
  int32_t *m_seq = mh + 5 * B, *m_pos = m_seq + T, *m_tseq = m_pos + T;
  int n_qtiles = 0, max_len = 0;
  {
    int t = 0;
    for (int b = 0; b < B; ++b) {
      m_len[b] = c->len[b];
      m_new[b] = bt->n_new[b];
      m_start[b] = t;
      m_off[b] = c->kv_off[b];
      m_cap[b] = c->cap_rows[b];
      for (int i = 0; i < bt->n_new[b]; ++i, ++t) {
        m_seq[t] = b;
        m_pos[t] = c->len[b] + i;
      }
      if (prefill) n_qtiles += (bt->n_new[b] + kPrefillQTile - 1) / kPrefillQTile;
      max_len = std::max(max_len, c->len[b] + bt->n_new[b]);
    }
  }
  int32_t* m_tq0 = m_tseq + n_qtiles;
  if (prefill) {
    int q = 0;
    for (int b = 0; b < B; ++b)
      for (int q0 = 0; q0 < bt->n_new[b]; q0 += kPrefillQTile, ++q) {
        m_tseq[q] = b;
        m_tq0[q] = q0;
      }
  }
  const size_t used_ints = (size_t)5 * B + 2 * (size_t)T + 2 * (size_t)n_qtiles;
  if (used_ints > c->meta_ints) return fail(c, SN_E_INVAL, "sn_step: index arrays overflow");
  // The index arrays are pulled from the pinned ring by a kernel, not by an asynchronous copy: a
  // copy engine serves its requests in order, so a copy that has to wait for the previous
  // iteration (stream order) would hold up every prefetch queued behind it on that engine.
  SN_HIP(c, launch_copy(c->meta_host_dev[ring], c->meta_dev, (used_ints * 4 + 15) / 16 * 16, c->compute));
  SN_HIP(c, hipEventRecord(c->ev_meta[ring], c->compute));
  c->meta_used[ring] = true;
  int32_t* md = c->meta_dev;
  StepIndex ix;
  ix.len_before = md;
  ix.n_new = md + B;
  ix.tok_start = md + 2 * B;
  ix.kv_off = md + 3 * B;
  ix.cap = md + 4 * B;
  ix.tok_seq = md + 5 * B;
  ix.tok_pos = ix.tok_seq + T;
  ix.tile_seq = ix.tok_pos + T;
  ix.tile_q0 = ix.tile_seq + n_qtiles;
  const int S = prefill ? 1 : attn_decode_splits(B, s.n_kv_heads, max_len);

  if (c->timing >= 2 && c->kev.empty()) {
    int rc = make_events(c, c->kev, L * kKernelsPerLayer * 2, true);
    if (rc) return rc;
  }
  c->last_kernel_class.assign(kKernelsPerLayer, 255);

  const uint64_t kv_used = (uint64_t)c->kv_used_tokens * kv_token_bytes(s);
  const bool fetch_kv = any_cached;             // prefill from empty caches produces the KV itself
  c->last_h2d_bytes = c->last_d2h_bytes = 0;
  c->last_preissued = 0;
  const int par = c->par;

  SN_HIP(c, hipEventRecord(c->ev_iter_start, c->compute));
  SN_HIP(c, launch_cast_in(s.dtype, bt->hidden_in, c->x32, (size_t)T * s.hidden, c->compute, c->flag_dev));
  Fold pending;

  for (int l = 0; l < L; ++l) {
    LayerState& ls = c->layers[l];
    if (c->timing >= 1 || ls.offloaded) SN_HIP(c, hipEventRecord(c->ev_layer[l], c->compute));
    // prefetches triggered by reaching this layer (paper Sec. 4.3: first layer of the group; eager
    // schedule: one group earlier, as soon as the staging slot is free)
    for (int o = l; o < L && o <= l + trigger_lead(c->N, c->sched); ++o) {
      LayerState& os = c->layers[o];
      if (!os.offloaded || os.trigger != l) continue;
      if (os.preissued) {            // already on its way (or here): issued during the previous iteration
        os.preissued = false;
        c->last_h2d_bytes += (int64_t)((os.w_host ? c->w_bytes : 0) + (os.kv_host ? kv_used : 0));
        ++c->last_preissued;
        continue;
      }
      int64_t bytes = 0;
      int rc = issue_load(c, o, par, fetch_kv, kv_used, &bytes);
      if (rc) return rc;
      c->last_h2d_bytes += bytes;
    }
    if (int rc = debug_delay(c, SN_DEBUG_DELAY_COMPUTE, c->compute)) return rc;
    uint8_t* base = ls.dev_w;
    uint8_t* kvbase = ls.dev_kv;
    uint8_t* mirror = nullptr;
    if (ls.offloaded) {
      SN_HIP(c, hipStreamWaitEvent(c->compute, c->ev_ready[par * L + l], 0));     // the fence "S" of Fig. 7
      SN_HIP(c, hipEventRecord(c->ev_after_wait[l], c->compute));
      if (ls.w_host) base = c->slot_w[ls.slot];
      if (ls.kv_host) kvbase = c->slot_kv[ls.slot];
      if (ls.kv_host && !prefill) mirror = ls.host_kv_dev;                   // decode: rows written through
    }
    // Whatever this layer's kernels write to the host slice (rows written through now, the slice copied back
    // after this prefill chunk) must land after an earlier write-back of the same slice has finished, or that
    // copy would overwrite the new rows with what the staging slot held.  Once the compute stream has waited,
    // everything enqueued later is ordered behind it (loads start from an event of the compute stream).
    if (ls.kv_host && ls.d2h_pending) {
      SN_HIP(c, hipStreamWaitEvent(c->compute, c->ev_d2h_end[l], 0));
      ls.d2h_pending = false;
    }
    int rc = run_layer(c, l, base, kvbase, mirror, ix, T, B, prefill, n_qtiles, S, pending);
    if (rc) return rc;
    if (ls.offloaded) {
      if (prefill && ls.kv_host) {
        SN_HIP(c, hipEventRecord(c->ev_done[l], c->compute));
        SN_HIP(c, hipStreamWaitEvent(c->d2h, c->ev_done[l], 0));
        if ((rc = debug_delay(c, SN_DEBUG_DELAY_D2H, c->d2h))) return rc;
        SN_HIP(c, hipEventRecord(c->ev_d2h_start[l], c->d2h));
        SN_HIP(c, hipMemcpyAsync(ls.host_kv, kvbase, kv_used, hipMemcpyDeviceToHost, c->d2h));
        SN_HIP(c, hipEventRecord(c->ev_d2h_end[l], c->d2h));
        ls.d2h_pending = true;
        SN_HIP(c, hipEventRecord(c->ev_slot_free[ls.slot], c->d2h));
        c->last_d2h_bytes += (int64_t)kv_used;
      } else {
        SN_HIP(c, hipEventRecord(c->ev_slot_free[ls.slot], c->compute));
        if (ls.kv_host) c->last_d2h_bytes += (int64_t)B * (int64_t)kv_token_bytes(s);
      }
      c->slot_free_valid[ls.slot] = true;
      // Continuous schedule, decode: the loads do not stop at the iteration boundary.  With K layers
      // on the host, the k-th one's completion releases what load k + min(2, K) waits for; when that
      // load belongs to the next iteration it is issued here, into the other event set.  It carries the
      // layer's weights and its whole KV slice (the rows this iteration wrote through included), which
      // is what any next iteration under the same placement and KV layout needs.
      if (c->sched == kSchedContinuous && !prefill) {
        const int K = offloaded_count(L, c->N), k = (l + 1) / c->N, ahead = std::min(2, K);
        if (k + ahead > K) {
          const int on = (k + ahead - K) * c->N - 1;
          int64_t bytes = 0;
          rc = issue_load(c, on, par ^ 1, true, kv_used, &bytes);
          if (rc) return rc;
          c->layers[on].preissued = true;
        }
      }
    }
  }
  SN_HIP(c, hipEventRecord(c->ev_layer[L], c->compute));
  if (pending.nsplit > 0)
    SN_HIP(c, launch_cast_out_fold(s.dtype, SN_F16, c->x32, hidden_out, T, s.hidden, pending, c->compute, c->flag_dev));
  else
    SN_HIP(c, launch_cast_out(s.dtype, c->x32, hidden_out, (size_t)T * s.hidden, c->compute, c->flag_dev));
  SN_HIP(c, hipEventRecord(c->ev_iter_end, c->compute));

  for (int b = 0; b < B; ++b) {
    c->len[b] += bt->n_new[b];
    kv->len[b] = c->len[b];
  }
  c->last_valid = true;
  c->last_par = par;
  c->par = par ^ 1;
  c->last_tokens = T;
  c->last_prefill = prefill;
  c->last_timing = c->timing;
  return SN_OK;
}

extern "C" int sn_read_hidden_f32(sn_ctx* c, void* dst, uint64_t dst_bytes) {
  if (!c || !dst) return fail(c, SN_E_INVAL, "sn_read_hidden_f32: null argument");
  if (!c->last_valid) return fail(c, SN_E_STATE, "sn_read_hidden_f32: no iteration has run under this placement");
  const uint64_t need = (uint64_t)c->last_tokens * c->shape.hidden * 4;
  if (dst_bytes < need) return fail(c, SN_E_INVAL, "sn_read_hidden_f32: destination holds %llu bytes, %llu needed",
                                    (unsigned long long)dst_bytes, (unsigned long long)need);
  SN_HIP(c, hipMemcpyAsync(dst, c->x32, need, hipMemcpyDeviceToDevice, c->compute));
  return SN_OK;
}

// =================================================================================
// stats
// =================================================================================
extern "C" int sn_set_timing(sn_ctx* c, int32_t level) {
  if (!c) return fail(nullptr, SN_E_INVAL, "null context");
  if (level < 0 || level > 2) return fail(c, SN_E_INVAL, "sn_set_timing: level must be 0, 1 or 2");
  c->timing = level;
  return SN_OK;
}

extern "C" int sn_set_kernel_timing_class(sn_ctx* c, int32_t kernel_class) {
  if (!c) return fail(nullptr, SN_E_INVAL, "null context");
  if (kernel_class < -1 || kernel_class > 7) return fail(c, SN_E_INVAL, "sn_set_kernel_timing_class: bad class");
  c->timing_class = kernel_class;
  return SN_OK;
}

extern "C" int sn_get_stats(sn_ctx* c, sn_step_stats* out) {
  if (!c || !out) return fail(c, SN_E_INVAL, "sn_get_stats: null argument");
  if (!c->last_valid) return fail(c, SN_E_STATE, "sn_get_stats: no iteration has run under this placement");
  int rc = sync_step(c);
  if (rc) return rc;
  std::memset(out, 0, sizeof *out);
  const int L = c->shape.n_layers;
  out->iter_ns = elapsed_ns(c->ev_iter_start, c->ev_iter_end);
  out->interval = c->N;
  out->resident_bytes = sn_resident_bytes(c, c->N);
  out->h2d_bytes = c->last_h2d_bytes;
  out->n_preissued = c->last_preissued;
  out->d2h_bytes = c->last_d2h_bytes;
  SN_HIP(c, hipMemcpy(&out->nonfinite, c->flag_dev, sizeof(int32_t), hipMemcpyDeviceToHost));
  for (int l = 0; l < L; ++l) {
    const LayerState& ls = c->layers[l];
    if (!ls.offloaded) continue;
    ++out->n_offloaded;
    out->h2d_ns += std::max<int64_t>(0, elapsed_ns(c->ev_copy_start[c->last_par * L + l], c->ev_ready[c->last_par * L + l]));
    out->stall_ns += std::max<int64_t>(0, elapsed_ns(c->ev_layer[l], c->ev_after_wait[l]));
    if (c->last_prefill && ls.kv_host) out->d2h_ns += std::max<int64_t>(0, elapsed_ns(c->ev_d2h_start[l], c->ev_d2h_end[l]));
  }
  out->hidden_fraction = out->h2d_ns > 0 ? 1.0 - (double)std::min(out->stall_ns, out->h2d_ns) / (double)out->h2d_ns : 1.0;
  if (c->last_timing >= 2 && !c->kev.empty()) {
    for (int l = 0; l < L; ++l)
      for (int k = 0; k < 8; ++k) {   // run_layer records 8 kernel slots
        const int cls = c->last_kernel_class[k];
        if (cls > 7) continue;            // this launch was not bracketed
        const int64_t ns = elapsed_ns(c->kev[((size_t)l * kKernelsPerLayer + k) * 2],
                                      c->kev[((size_t)l * kKernelsPerLayer + k) * 2 + 1]);
        if (ns >= 0) {
          out->kernel_ns[cls] += ns;
          out->kernel_calls[cls] += 1;
        }
      }
  }
  return SN_OK;
}

extern "C" int sn_time_kernel_class(sn_ctx* c, int32_t kernel_class, int32_t batch, int32_t reps, int64_t* total_ns,
                                    int32_t* launches) {
  if (!c || !total_ns || !launches) return fail(c, SN_E_INVAL, "sn_time_kernel_class: null argument");
  if (!c->placed) return fail(c, SN_E_STATE, "sn_time_kernel_class before sn_place");
  if (batch < 1 || batch > kMaxDecodeRows || batch > c->shape.max_batch || reps < 1 || reps > 1000)
    return fail(c, SN_E_INVAL, "sn_time_kernel_class: bad batch or reps");
  const sn_model_shape& s = c->shape;
  const PackedLayout& p = c->pl;
  const int h = s.hidden, F = s.ffn, qd = s.n_q_heads * s.head_dim;
  int rc = sync_all(c);
  if (rc) return rc;
  int n = 0;
  SN_HIP(c, hipEventRecord(c->ev_iter_start, c->compute));
  for (int r = 0; r < reps; ++r)
    for (const LayerState& ls : c->layers) {
      if (!ls.dev_w) continue;
      auto at = [&](uint64_t off) -> const void* { return off == kNone ? nullptr : ls.dev_w + off; };
      hipError_t e;
      switch (kernel_class) {
        case SN_K_QKV:
          if (const int qs = c->qkv_part32 ? gemm_qkv_splits(batch, p.n_qkv, h) : 0)
            e = launch_gemm_skinny(SN_F16, EPI_PART32, at(p.wqkv), c->u16, at(p.bqkv), c->qkv_part32, batch, p.n_qkv, h, c->compute, qs, kXPacked);
          else
            e = launch_gemm_skinny(SN_F16, EPI_STORE16, at(p.wqkv), c->u16, at(p.bqkv), c->qkv16, batch, p.n_qkv, h, c->compute, 1, kXPacked);
          break;
        case SN_K_OPROJ:
          e = launch_gemm_skinny(SN_F16, EPI_PART32, at(p.wo), c->attn16, nullptr, c->part32, batch, h, qd, c->compute,
                                 gemm_skinny_splits(batch, h, qd), kXPacked);
          break;
        case SN_K_FFN_UP:
          e = launch_gemm_skinny(SN_F16, s.act == SN_ACT_SWIGLU ? EPI_SWIGLU16 : EPI_GELU16, at(p.wup), c->u16, at(p.bup),
                                 c->act16, batch, p.n_up, h, c->compute, 1, kXPacked | kOutPacked);
          break;
        case SN_K_FFN_DOWN:
          e = launch_gemm_skinny(SN_F16, EPI_PART32, at(p.wd), c->act16, nullptr, c->part32, batch, h, F, c->compute,
                                 gemm_skinny_splits(batch, h, F), kXPacked);
          break;
        default:
          return fail(c, SN_E_INVAL, "sn_time_kernel_class: only the four projection classes can be timed alone");
      }
      if (e != hipSuccess) return fail(c, SN_E_HIP, "sn_time_kernel_class: %s", hipGetErrorString(e));
      ++n;
    }
  SN_HIP(c, hipEventRecord(c->ev_iter_end, c->compute));
  SN_HIP(c, hipStreamSynchronize(c->compute));
  if (n == 0) return fail(c, SN_E_STATE, "sn_time_kernel_class: no GPU-resident layer under this placement");
  *total_ns = elapsed_ns(c->ev_iter_start, c->ev_iter_end);
  *launches = n;
  c->last_valid = false;
  return SN_OK;
}

extern "C" int sn_get_layer_times(sn_ctx* c, int64_t* compute_ns, int64_t* stall_ns, int64_t* h2d_ns) {
  if (!c) return fail(nullptr, SN_E_INVAL, "null context");
  if (!c->last_valid) return fail(c, SN_E_STATE, "sn_get_layer_times: no iteration has run under this placement");
  if (c->last_timing < 1) return fail(c, SN_E_STATE, "sn_get_layer_times: needs timing level >= 1 during the step");
  int rc = sync_step(c);
  if (rc) return rc;
  const int L = c->shape.n_layers;
  for (int l = 0; l < L; ++l) {
    const LayerState& ls = c->layers[l];
    if (compute_ns) compute_ns[l] = elapsed_ns(ls.offloaded ? c->ev_after_wait[l] : c->ev_layer[l], c->ev_layer[l + 1]);
    if (stall_ns) stall_ns[l] = ls.offloaded ? std::max<int64_t>(0, elapsed_ns(c->ev_layer[l], c->ev_after_wait[l])) : 0;
    if (h2d_ns) h2d_ns[l] = ls.offloaded ? elapsed_ns(c->ev_copy_start[c->last_par * L + l], c->ev_ready[c->last_par * L + l]) : 0;
  }
  return SN_OK;
}

// =================================================================================
// profiler and picker (paper Sec. 4.4)
// =================================================================================
static int64_t median_of(std::vector<int64_t> v) {
  std::sort(v.begin(), v.end());
  return v[v.size() / 2];
}

extern "C" int sn_profile_layers(sn_ctx* c, int32_t is_prefill, int32_t batch, int32_t seq, int32_t reps,
                                 int64_t* tc_ns, int64_t* tx_ns) {
  if (!c) return fail(nullptr, SN_E_INVAL, "sn_profile_layers: null context");
  if (!c->placed) return fail(c, SN_E_STATE, "sn_profile_layers before sn_place");
  const sn_model_shape& s = c->shape;
  const int L = s.n_layers;
  if (batch < 1 || batch > s.max_batch || seq < 1 || reps < 1 || reps > 1000)
    return fail(c, SN_E_INVAL, "sn_profile_layers: bad batch/seq/reps");
  if (!is_prefill && batch > kMaxDecodeRows) return fail(c, SN_E_INVAL, "sn_profile_layers: decode batch above %d", kMaxDecodeRows);
  const int cap1 = is_prefill ? seq : seq + 1;
  if ((int64_t)cap1 * batch > (int64_t)s.max_batch * s.max_seq)
    return fail(c, SN_E_INVAL, "sn_profile_layers: batch*seq exceeds the context's KV capacity");
  const int64_t T = is_prefill ? (int64_t)batch * seq : batch;
  if (T > c->max_tokens) return fail(c, SN_E_INVAL, "sn_profile_layers: too many tokens for max_tokens");

  int rc = sync_all(c);
  if (rc) return rc;
  // The iterations run here are measurements, each followed by a reset: nothing is issued ahead.
  struct SchedGuard {
    sn_ctx* c;
    int saved;
    ~SchedGuard() { c->sched = saved; }
  } guard{c, c->sched};
  if (c->sched == kSchedContinuous) c->sched = kSchedEager;
  std::vector<int32_t> caps(batch, cap1), n_new(batch, is_prefill ? seq : 1), lens(batch, 0);
  if ((rc = sn_kv_reset(c, batch, caps.data()))) return rc;

  void *hin = nullptr, *hout = nullptr;
  const size_t hbytes = (size_t)T * s.hidden * 2;
  SN_HIP(c, hipMalloc(&hin, hbytes));
  if (hipMalloc(&hout, hbytes) != hipSuccess) {
    (void)hipFree(hin);
    return fail(c, SN_E_NOMEM, "sn_profile_layers: device allocation failed");
  }
  const int saved_timing = c->timing;
  c->timing = 1;
  std::vector<std::vector<int64_t>> samples(L);
  std::vector<int64_t> tcur(L);
  sn_batch bt{batch, is_prefill ? 1 : 0, n_new.data(), hin};
  sn_kv kvh{lens.data()};
  rc = SN_OK;
  hipError_t he = launch_fill_hash(s.dtype, hin, (size_t)T * s.hidden, 12345u, c->compute);
  if (he != hipSuccess) rc = fail(c, SN_E_HIP, "fill: %s", hipGetErrorString(he));
  for (int r = 0; r < reps + 1 && rc == SN_OK; ++r) {   // first pass is a warm-up
    for (int b = 0; b < batch; ++b) c->len[b] = lens[b] = is_prefill ? 0 : seq;
    rc = sn_step(c, &bt, &kvh, hout);
    if (rc) break;
    rc = sn_get_layer_times(c, tcur.data(), nullptr, nullptr);
    if (rc) break;
    if (r > 0)
      for (int l = 0; l < L; ++l) samples[l].push_back(tcur[l]);
  }
  c->timing = saved_timing;
  if (rc) {
    (void)hipFree(hin);
    (void)hipFree(hout);
    return rc;
  }
  int64_t iter_est = 0;
  for (int l = 0; l < L; ++l) {
    c->prof_tc[l] = median_of(samples[l]);
    iter_est += c->prof_tc[l];
  }

  // Transfer of each layer's state -- the part of it that is kept on the host when the layer is
  // host-resident (weights; + KV prefix when decoding) -- timed while the
  // compute stream runs iterations of the same kind: that is the condition under which
  // prefetches run, and copies are a little slower then than on an idle GPU.
  // Destination: a scratch state of its own (the staging slots hold only the part that travels).
  uint8_t* dst = nullptr;
  const bool temp = true;
  if (hipMalloc((void**)&dst, c->state_bytes) != hipSuccess) {
    (void)hipFree(hin);
    (void)hipFree(hout);
    return fail(c, SN_E_NOMEM, "sn_profile_layers: device allocation failed");
  }
  const bool copy_w = weights_travel(c->what);
  const uint64_t kv_used = (is_prefill || !kv_travels(c->what)) ? 0 : (uint64_t)c->kv_used_tokens * kv_token_bytes(s);
  uint8_t* kv_src_tmp = nullptr;
  int64_t tx_est = 0;
  const int tx_reps = std::min(reps, 3);
  // sources: the layer's own pinned master / KV slice where it has one, else pinned stand-ins of the same size
  std::vector<const uint8_t*> w_srcs(L), kv_srcs(L, nullptr);
  for (int l = 0; l < L && rc == SN_OK; ++l) {
    LayerState& ls = c->layers[l];
    kv_srcs[l] = ls.host_kv;
    if (kv_used && !kv_srcs[l]) {   // resident layer: time the same bytes from a pinned scratch slice
      if (!kv_src_tmp) {
        if (hipHostMalloc((void**)&kv_src_tmp, c->kv_bytes, hipHostMallocDefault) != hipSuccess) {
          rc = fail(c, SN_E_NOMEM, "sn_profile_layers: pinned allocation failed");
          break;
        }
        std::memset(kv_src_tmp, 0, c->kv_bytes);
      }
      kv_srcs[l] = kv_src_tmp;
    }
    w_srcs[l] = ls.host_w;
    if (!w_srcs[l]) {               // no host master (the layer lives on the GPU): same bytes from the staging record
      if (ensure_stage(c)) {
        rc = SN_E_NOMEM;
        break;
      }
      w_srcs[l] = c->stage_w;
    }
  }
  auto timed_copy = [&](int l) -> hipError_t {
    hipError_t e = hipEventRecord(c->ev_copy_start[l], c->h2d);
    if (e == hipSuccess && copy_w) e = hipMemcpyAsync(dst, w_srcs[l], c->w_bytes, hipMemcpyHostToDevice, c->h2d);
    if (e == hipSuccess && kv_used) e = hipMemcpyAsync(dst + c->w_bytes, kv_srcs[l], kv_used, hipMemcpyHostToDevice, c->h2d);
    if (e == hipSuccess) e = hipEventRecord(c->ev_ready[l], c->h2d);
    return e;
  };
  auto sync_streams = [&]() -> hipError_t {
    hipError_t e = hipStreamSynchronize(c->h2d);
    if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
    if (e == hipSuccess) e = hipStreamSynchronize(c->d2h);
    return e;
  };
  if (rc == SN_OK) {                // idle-GPU warm-up copy: gives the estimate, not a sample
    hipError_t e = timed_copy(0);
    if (e == hipSuccess) e = sync_streams();
    if (e != hipSuccess) rc = fail(c, SN_E_HIP, "sn_profile_layers: transfer timing: %s", hipGetErrorString(e));
    else tx_est = std::max<int64_t>(1, elapsed_ns(c->ev_copy_start[0], c->ev_ready[0]));
  }
  // A round: enough iterations on the compute stream to outlast the copies, then as many layers' copies,
  // back to back on the copy stream, as fit under them (one when an iteration is shorter than a copy, as in
  // decoding; many when it is much longer, as in prefill -- which keeps the profile of a large prefill to
  // seconds instead of minutes).
  const int64_t iter_ns = std::max<int64_t>(1, iter_est);
  const int busy = (int)std::min<int64_t>(64, (tx_est + tx_est / 4 + iter_ns - 1) / iter_ns + 1);
  const int per_round = (int)std::max<int64_t>(1, std::min<int64_t>(L, (int64_t)busy * iter_ns / (tx_est + tx_est / 4)));
  std::vector<std::vector<int64_t>> tx_samples(L);
  for (int r = 0; r < tx_reps && rc == SN_OK; ++r)
    for (int l0 = 0; l0 < L && rc == SN_OK; l0 += per_round) {
      const int l1 = std::min(L, l0 + per_round);
      for (int k = 0; k < busy && rc == SN_OK; ++k) {
        for (int b = 0; b < batch; ++b) c->len[b] = lens[b] = is_prefill ? 0 : seq;
        rc = sn_step(c, &bt, &kvh, hout);
      }
      if (rc) break;
      hipError_t e = hipSuccess;
      for (int l = l0; l < l1 && e == hipSuccess; ++l) e = timed_copy(l);
      if (e == hipSuccess) e = sync_streams();
      if (e != hipSuccess) {
        rc = fail(c, SN_E_HIP, "sn_profile_layers: transfer timing: %s", hipGetErrorString(e));
        break;
      }
      for (int l = l0; l < l1; ++l) tx_samples[l].push_back(elapsed_ns(c->ev_copy_start[l], c->ev_ready[l]));
    }
  for (int l = 0; l < L && rc == SN_OK; ++l) c->prof_tx[l] = median_of(tx_samples[l]);
  (void)hipFree(hin);
  (void)hipFree(hout);
  if (kv_src_tmp) (void)hipHostFree(kv_src_tmp);
  if (temp) (void)hipFree(dst);
  if (rc) return rc;

  for (int b = 0; b < batch; ++b) c->len[b] = 0;
  c->last_valid = false;
  c->has_profile = true;
  if (tc_ns) std::copy(c->prof_tc.begin(), c->prof_tc.end(), tc_ns);
  if (tx_ns) std::copy(c->prof_tx.begin(), c->prof_tx.end(), tx_ns);
  return SN_OK;
}

extern "C" int sn_pick_interval(sn_ctx* c, double slo_ms, int32_t* N_out) {
  if (!c || !N_out) return fail(c, SN_E_INVAL, "sn_pick_interval: null argument");
  if (!c->has_profile) return fail(c, SN_E_STATE, "sn_pick_interval before sn_profile_layers");
  if (!(slo_ms > 0)) return fail(c, SN_E_INVAL, "sn_pick_interval: SLO must be positive");
  const int64_t slo_ns = (int64_t)std::llround(slo_ms * 1.0e6);
  const int L = c->shape.n_layers;
  const int rc = sn_pick_interval_from_times_sched(L, c->prof_tc.data(), c->prof_tx.data(), slo_ns, sn_max_interval(c),
                                                   c->sched, N_out);
  if (rc) {
    c->err = g_err;
    return rc;
  }
  // The two staging slots make an interval close to L cost more device memory than
  // keeping the whole model resident.  If the pick does not fit although "no
  // offloading" does (the only way minimum <= maximum can still not fit), run without
  // offloading: its iteration time is no longer and it is within capacity.
  if (c->budget && sn_resident_bytes(c, *N_out) > c->budget) *N_out = L + 1;
  return SN_OK;
}

extern "C" int sn_refine_interval(sn_ctx* c, int32_t N, int32_t* N_out) {
  if (!c || !N_out) return fail(c, SN_E_INVAL, "sn_refine_interval: null argument");
  if (!c->has_profile) return fail(c, SN_E_STATE, "sn_refine_interval before sn_profile_layers");
  const int rc = sn_refine_interval_from_times(c->shape.n_layers, c->prof_tc.data(), c->prof_tx.data(), N, c->sched, N_out);
  if (rc) c->err = g_err;
  return rc;
}

// =================================================================================
// entry point for callers that cannot allocate
// =================================================================================
extern "C" int sn_k_attn_decode_static(int32_t dtype, const void* qkv16, const void* kv, const int32_t* len_before,
                                       const int32_t* kv_off, const int32_t* cap, void* out16, int32_t B, int32_t Hq,
                                       int32_t Hkv, int32_t d, int32_t S, int32_t max_len, int32_t packed_out,
                                       void* stream) {
  if ((dtype != SN_F16 && dtype != SN_BF16) || !qkv16 || !kv || !len_before || !kv_off || !cap || !out16 || B < 0 ||
      Hq < 1 || Hkv < 1 || Hq % Hkv || (d != 64 && d != 128) || S < 0 || S > 16)
    return fail(nullptr, SN_E_INVAL, "sn_k_attn_decode_static: bad argument");
  if (S == 0) {
    if (max_len < 1) return fail(nullptr, SN_E_INVAL, "sn_k_attn_decode_static: S == 0 needs max_len");
    S = attn_decode_splits(B, Hkv, max_len);
  }
  // the partial results of the key ranges: [B][Hq][S][d+2] fp32, every element written before it is read
  const uint64_t need = S > 1 ? (uint64_t)B * Hq * S * (d + 2) * sizeof(float) : 0;
  if (need > SN_K_STATIC_SCRATCH_BYTES)
    return fail(nullptr, SN_E_INVAL,
                "sn_k_attn_decode_static: %d sequences x %d heads x %d key ranges need %llu bytes of partial results, the "
                "static buffer holds %llu; use sn_k_attn_decode with a buffer of your own",
                B, Hq, S, (unsigned long long)need, (unsigned long long)SN_K_STATIC_SCRATCH_BYTES);
  void* part = nullptr;
  const hipError_t es = static_scratch(&part);
  if (es != hipSuccess) return fail(nullptr, SN_E_HIP, "sn_k_attn_decode_static: static scratch buffer: %s", hipGetErrorString(es));
  StepIndex ix{};
  ix.len_before = len_before;
  ix.kv_off = kv_off;
  ix.cap = cap;
  const hipError_t e = launch_attn_decode(dtype, qkv16, kv, ix, out16, static_cast<float*>(part), B, Hq, Hkv, d, S,
                                          (hipStream_t)stream, packed_out != 0);
  if (e != hipSuccess)
    return fail(nullptr, e == hipErrorInvalidValue ? SN_E_INVAL : SN_E_HIP, "sn_k_attn_decode_static: %s", hipGetErrorString(e));
  return SN_OK;
}
