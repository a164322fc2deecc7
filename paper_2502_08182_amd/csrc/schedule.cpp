// Placement map, prefetch triggers, the iteration timeline and the interval picker.
// Host only, exact int64 arithmetic.
//
// Paper: an offloading interval of i keeps, for every i layers, the last one on the
// host (Sec. 4.3); its load is issued when compute reaches the first layer of that
// group, and a synchronisation point precedes the offloaded layer (Fig. 7); the
// optimal interval is the smallest one that meets the SLO (Sec. 4.3, 4.4) and must not
// exceed the maximum allowed by GPU capacity (Sec. 4.5).
#include "schedule.h"

#include <algorithm>
#include <vector>

namespace sn {

int offloaded_count(int L, int N) { return (N >= 1 && N <= L) ? L / N : 0; }

bool is_offloaded(int L, int N, int l) { return N >= 1 && N <= L && (l + 1) % N == 0; }

int trigger_lead(int N, int sched) {
  // paper: first layer of the group; one layer ahead when every layer is offloaded (N == 1).
  // eager: one group earlier -- the staging slot of the k-th offloaded layer is free once the
  // (k-2)-th has been computed, so its load can be issued at the layer after that one.
  // continuous: within an iteration as eager (what it adds happens at the iteration boundary).
  return sched != kSchedPaper ? 2 * N - 1 : (N > 1 ? N - 1 : 1);
}

int trigger_of(int N, int o, int sched) {
  const int lead = trigger_lead(N, sched);
  return o >= lead ? o - lead : 0;
}

// Steady state of back-to-back iterations whose loads run on across the iteration boundary.
// Loads are numbered through all iterations; load g (iteration g / K, g % K-th offloaded layer) is
// handed to the copy stream when the layer of load g - min(2, K) has been computed (its staging slot
// is free then; with a single offloaded layer, its KV rows of the previous iteration are written
// then), the first min(2, K) at time zero.  The copy stream is FIFO in that order, so each load's
// arrival follows from the previous load's arrival and that one compute-finish time, both of
// which are known by the time compute reaches the load's own layer.  Reports the longer of the
// last two of kContinuousIterations iterations and the stalls of the last one.
static int64_t continuous_time(int L, const int64_t* tc, const int64_t* tx, int N, int64_t* stall_total) {
  const int K = offloaded_count(L, N);
  const int m = std::min(2, K);
  const int total = kContinuousIterations * K;
  std::vector<int64_t> arrive(total), finish(total);
  int64_t now = 0, last = 0, before_last = 0, stalls = 0;
  for (int it = 0, g = 0; it < kContinuousIterations; ++it) {
    const int64_t begin = now;
    stalls = 0;
    for (int l = 0; l < L; ++l) {
      if (is_offloaded(L, N, l)) {
        const int64_t handed_over = g < m ? 0 : finish[g - m];
        arrive[g] = std::max(g ? arrive[g - 1] : 0, handed_over) + tx[l];
        const int64_t wait = std::max<int64_t>(0, arrive[g] - now);
        stalls += wait;
        now += wait + tc[l];
        finish[g++] = now;
      } else {
        now += tc[l];
      }
    }
    before_last = last;
    last = now - begin;
  }
  if (stall_total) *stall_total = stalls;
  return std::max(last, before_last);
}

int64_t iteration_time(int L, const int64_t* tc, const int64_t* tx, int N, int64_t* stall_total, int sched) {
  if (sched == kSchedContinuous && offloaded_count(L, N) > 0) return continuous_time(L, tc, tx, N, stall_total);
  // Walk the offloaded layers in order.  `now` is the compute stream's clock at the
  // start of the layer under consideration, `copy_idle` the time the (single, FIFO)
  // copy stream runs dry.  Prefix sums give the clock at any trigger layer without
  // stepping through resident layers one by one; stalls shift everything after them.
  std::vector<int64_t> pre(L + 1, 0);
  for (int l = 0; l < L; ++l) pre[l + 1] = pre[l] + tc[l];
  int64_t shift = 0;        // total stall so far
  int64_t copy_idle = 0;
  int64_t stalls = 0;
  const int K = offloaded_count(L, N);
  // Stalls at offloaded layers strictly before a trigger layer delay that trigger.
  // Offloaded layers are visited in increasing order.  A trigger g_k never lies beyond the
  // previous offloaded layer o_{k-1}; when it coincides with it (N == 1) it fires at the
  // *start* of o_{k-1}, i.e. before that layer's own stall; with the eager schedule it is the
  // layer right after o_{k-2}, whose stall is already part of the shift recorded for it.
  std::vector<int64_t> shift_before(L + 1, 0);   // stall accumulated before layer l starts waiting
  int next_fill = 0;
  for (int k = 1; k <= K; ++k) {
    const int o = k * N - 1;
    const int g = trigger_of(N, o, sched);
    for (; next_fill <= o; ++next_fill) shift_before[next_fill] = shift;
    const int64_t issue = pre[g] + shift_before[g];
    const int64_t begin = std::max(copy_idle, issue);
    copy_idle = begin + tx[o];
    const int64_t arrive_at_fence = pre[o] + shift;
    const int64_t wait = std::max<int64_t>(0, copy_idle - arrive_at_fence);
    stalls += wait;
    shift += wait;
  }
  if (stall_total) *stall_total = stalls;
  return pre[L] + shift;
}

int min_interval(int L, const int64_t* tc, const int64_t* tx, int64_t slo, int sched) {
  // Measured layer times need not make T(N) monotone in N, so every N is tried.
  for (int N = 1; N <= L; ++N)
    if (iteration_time(L, tc, tx, N, nullptr, sched) <= slo) return N;
  int64_t all = 0;
  for (int l = 0; l < L; ++l) all += tc[l];
  return all <= slo ? L + 1 : -1;
}

// Sec. 4.3 / 4.4 rank intervals by how many layers they offload; intervals with the same floor(L / N) offload the same
// layers' worth of host memory and leave the same GPU footprint, and the paper does not choose between them.  Of
// those, the shortest iteration (the smallest interval on a tie); N itself is a candidate, so the result is never slower.
int refine_interval(int L, const int64_t* tc, const int64_t* tx, int N, int sched) {
  if (N > L) return N;
  const int K = offloaded_count(L, N);
  int best = N;
  int64_t best_t = iteration_time(L, tc, tx, N, nullptr, sched);
  for (int cand = N + 1; cand <= L && offloaded_count(L, cand) == K; ++cand) {
    const int64_t t = iteration_time(L, tc, tx, cand, nullptr, sched);
    if (t < best_t) best = cand, best_t = t;
  }
  return best;
}

uint64_t resident_bytes(int L, int N, uint64_t state, uint64_t slot, uint64_t fixed) {
  const int K = offloaded_count(L, N);
  return (uint64_t)(L - K) * state + (K ? 2 * slot : 0) + fixed;
}

// What a host-resident layer leaves on the GPU, and what a staging slot holds, when the layer keeps on
// the host its whole state (0), only its weights (1) or only its KV slice (2).
static uint64_t part_left_behind(uint64_t weight_bytes, uint64_t kv_bytes, int what) {
  return what == 1 ? kv_bytes : what == 2 ? weight_bytes : 0;
}

uint64_t resident_bytes_of(int L, int N, uint64_t weight_bytes, uint64_t kv_bytes, uint64_t fixed, int what) {
  const int K = offloaded_count(L, N);
  const uint64_t stays = part_left_behind(weight_bytes, kv_bytes, what);
  const uint64_t travels = weight_bytes + kv_bytes - stays;
  return (uint64_t)(L - K) * (weight_bytes + kv_bytes) + (uint64_t)K * stays + (K ? 2 * travels : 0) + fixed;
}

int max_interval_of(int L, uint64_t budget, uint64_t weight_bytes, uint64_t kv_bytes, uint64_t fixed, int what) {
  if (budget == 0) return L + 1;
  int best = 0;
  for (int N = 1; N <= L + 1; ++N)
    if (resident_bytes_of(L, N, weight_bytes, kv_bytes, fixed, what) <= budget) best = N;
  return best;
}

uint64_t max_tokens(int L, int N, uint64_t weight_bytes, uint64_t kv_token_bytes, uint64_t fixed, uint64_t budget, int what) {
  // The footprint is linear in the token count t: copies of the weights and copies of the KV slice
  // (t * kv_token_bytes each).  GPU-resident layers hold both; a host-resident layer holds the part it
  // leaves behind; the two staging slots (when anything is offloaded) hold the part that travels.
  const int K = offloaded_count(L, N);
  unsigned __int128 w_copies = (unsigned __int128)(L - K), kv_copies = w_copies;
  if (K) {
    if (what == 1) { kv_copies += K; w_copies += 2; }
    else if (what == 2) { w_copies += K; kv_copies += 2; }
    else { w_copies += 2; kv_copies += 2; }
  }
  const unsigned __int128 base = w_copies * weight_bytes + fixed;
  if (kv_token_bytes == 0 || kv_copies == 0 || base > budget) return 0;
  const unsigned __int128 t = ((unsigned __int128)budget - base) / (kv_copies * kv_token_bytes);
  return t > (unsigned __int128)UINT64_MAX ? UINT64_MAX : (uint64_t)t;
}

int max_interval(int L, uint64_t budget, uint64_t state, uint64_t slot, uint64_t fixed) {
  if (budget == 0) return L + 1;
  int best = 0;
  for (int N = 1; N <= L + 1; ++N)
    if (resident_bytes(L, N, state, slot, fixed) <= budget) best = N;
  return best;
}

int32_t paper_rule(int L, int64_t t_trans, int64_t slo) {
  if (t_trans <= 0) return 1;
  const int64_t l_off = slo / t_trans;
  return (int32_t)(L / (l_off + 1) + 1);
}

}  // namespace sn
