// The per-bus bandwidth coordinator (paper Sec. 4.5, Fig. 8): exact integer arithmetic.
//
// The objective and the constraint depend on an instance's interval only through the number of
// layers it offloads, K = floor(L / N), which takes O(sqrt(L)) distinct values; among the
// intervals with the same K the tie-break (lexicographically smallest tuple) wants the smallest.
// So each instance contributes one candidate per distinct K in its range, in ascending interval
// order, and the search is a depth-first enumeration of those with two cuts: the bandwidth
// already committed, and a bound on the host memory still attainable.
#include <algorithm>
#include <vector>

#include "../../include/sn_coord.h"

namespace {

struct Cand {
  int32_t N;
  uint64_t mem, rate;
};

struct Search {
  std::vector<std::vector<Cand>> cands;   // per instance, ascending N (so descending mem)
  std::vector<unsigned __int128> rest;    // best host memory attainable by instances i..n-1
  unsigned __int128 bandwidth = 0;
  std::vector<int32_t> cur, best;
  unsigned __int128 best_mem = 0, best_rate = 0;
  bool found = false;

  void go(size_t i, unsigned __int128 mem, unsigned __int128 rate) {
    if (i == cands.size()) {
      if (!(rate < bandwidth)) return;
      const bool better = !found || mem > best_mem || (mem == best_mem && rate < best_rate) ||
                          (mem == best_mem && rate == best_rate && cur < best);
      if (better) {
        found = true;
        best = cur;
        best_mem = mem;
        best_rate = rate;
      }
      return;
    }
    if (found && mem + rest[i] < best_mem) return;   // cannot reach the best any more (ties must still be explored)
    for (const Cand& c : cands[i]) {
      if (!(rate + c.rate < bandwidth)) continue;    // rates only add up: already too much
      cur[i] = c.N;
      go(i + 1, mem + c.mem, rate + c.rate);
    }
  }
};

bool bad(const sn_coord_instance* g) { return !g || g->n_layers < 1 || g->iter_ns <= 0 || g->reserved != 0; }

}  // namespace

extern "C" int32_t sn_coord_offloaded(const sn_coord_instance* g, int32_t N) {
  if (bad(g) || N < 1 || N > g->n_layers) return 0;
  return g->n_layers / N;
}

extern "C" uint64_t sn_coord_host_bytes(const sn_coord_instance* g, int32_t N) {
  return (uint64_t)sn_coord_offloaded(g, N) * (g ? g->mem_per_layer : 0);
}

extern "C" uint64_t sn_coord_rate(const sn_coord_instance* g, int32_t N) {
  if (bad(g)) return 0;
  const unsigned __int128 b = (unsigned __int128)sn_coord_host_bytes(g, N) * 1000000000u / (unsigned __int128)g->iter_ns;
  return b > (unsigned __int128)UINT64_MAX ? UINT64_MAX : (uint64_t)b;
}

extern "C" int sn_coord_adjust(const sn_coord_instance* inst, int32_t n, uint64_t bandwidth, int32_t* N_out,
                               uint64_t* host_bytes_out, uint64_t* rate_out) {
  if (!inst || !N_out || n < 1 || n > SN_COORD_MAX_INSTANCES) return SN_E_INVAL;
  for (int i = 0; i < n; ++i)
    if (bad(&inst[i]) || inst[i].n_min < 1 || inst[i].n_max < 0) return SN_E_INVAL;
  Search s;
  s.bandwidth = bandwidth;
  s.cands.resize(n);
  for (int i = 0; i < n; ++i) {
    const sn_coord_instance& g = inst[i];
    const int32_t hi = std::min(g.n_max, g.n_layers + 1);
    if (g.n_min > hi) return SN_E_INFEASIBLE;        // Fig. 8, first check: the SLO cannot be met within capacity
    int32_t last_k = -1;
    for (int32_t N = g.n_min; N <= hi; ++N) {
      const int32_t k = sn_coord_offloaded(&g, N);
      if (k == last_k) continue;                     // same layers offloaded as a smaller interval
      last_k = k;
      s.cands[i].push_back(Cand{N, sn_coord_host_bytes(&g, N), sn_coord_rate(&g, N)});
    }
  }
  s.rest.assign(n + 1, 0);
  for (int i = n - 1; i >= 0; --i) s.rest[i] = s.rest[i + 1] + s.cands[i].front().mem;
  s.cur.assign(n, 0);
  s.go(0, 0, 0);
  if (!s.found) return SN_E_INFEASIBLE;
  std::copy(s.best.begin(), s.best.end(), N_out);
  if (host_bytes_out) *host_bytes_out = s.best_mem > (unsigned __int128)UINT64_MAX ? UINT64_MAX : (uint64_t)s.best_mem;
  if (rate_out) *rate_out = s.best_rate > (unsigned __int128)UINT64_MAX ? UINT64_MAX : (uint64_t)s.best_rate;
  return SN_OK;
}
