// Host-only schedule arithmetic (placement, timeline, picker, capacity bound).
#pragma once
#include <stdint.h>

namespace sn {
int offloaded_count(int L, int N);
bool is_offloaded(int L, int N, int l);
constexpr int kSchedPaper = 0, kSchedEager = 1, kSchedContinuous = 2;   // when the load of an offloaded layer is issued
constexpr int kContinuousIterations = 16;         // iterations walked to the continuous schedule's steady state
int trigger_lead(int N, int sched);               // layers between the trigger and the offloaded layer
int trigger_of(int N, int offloaded_layer, int sched = kSchedPaper);
int64_t iteration_time(int L, const int64_t* tc, const int64_t* tx, int N, int64_t* stall_total, int sched = kSchedPaper);
int min_interval(int L, const int64_t* tc, const int64_t* tx, int64_t slo, int sched = kSchedPaper);   // -1: none
int refine_interval(int L, const int64_t* tc, const int64_t* tx, int N, int sched = kSchedPaper);     // fastest interval offloading as many layers as N
uint64_t resident_bytes(int L, int N, uint64_t state, uint64_t slot, uint64_t fixed);
int max_interval(int L, uint64_t budget, uint64_t state, uint64_t slot, uint64_t fixed);
// `what`: the part of a host-resident layer's state kept on the host -- 0 whole state, 1 weights, 2 KV slice
uint64_t resident_bytes_of(int L, int N, uint64_t weight_bytes, uint64_t kv_bytes, uint64_t fixed, int what);
int max_interval_of(int L, uint64_t budget, uint64_t weight_bytes, uint64_t kv_bytes, uint64_t fixed, int what);
uint64_t max_tokens(int L, int N, uint64_t weight_bytes, uint64_t kv_token_bytes, uint64_t fixed, uint64_t budget, int what = 0);
int32_t paper_rule(int L, int64_t t_trans, int64_t slo);
}  // namespace sn
