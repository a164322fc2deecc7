// The analyzer's performance record (paper Sec. 4.4): cells of measured per-layer times
// keyed by (phase, batch, seq), the optimal interval of a cell for a latency bound, the
// conservative nearest-combination lookup, a Table-1 view and JSON persistence.
// Host-only; the one entry point that touches the GPU is sn_record_profile, which only
// calls the public profiler.
#include <cctype>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <set>
#include <string>
#include <tuple>
#include <vector>

#include "../../include/sn_record.h"
#include "schedule.h"

namespace {

struct Cell {
  std::vector<int64_t> tc, tx;
  int32_t n_max = 0;
};

using Key = std::tuple<int32_t, int32_t, int32_t>;   // phase, batch, seq

}  // namespace

struct sn_record {
  int32_t L = 0;
  int64_t step = 0;
  std::map<Key, Cell> cells;
};

namespace {

bool bad_phase(int32_t p) { return p != SN_PHASE_DECODE && p != SN_PHASE_PREFILL; }

// Latency bound of a cell in ns, or -1 for a bad kind / value.
int64_t bound_ns(const sn_record* r, const Cell& c, int32_t kind, int64_t value) {
  if (value < 0) return -1;
  if (kind == SN_SLO_REL_PERMILLE) {
    __int128 sum = 0;
    for (int64_t v : c.tc) sum += v;
    const __int128 b = sum * value / 1000;
    return b > (__int128)INT64_MAX ? INT64_MAX : (int64_t)b;
  }
  if (kind == SN_SLO_ABS_NS) return r->step > 0 ? value - value % r->step : value;
  return -1;
}

// SN_OK + *N, or SN_E_INFEASIBLE.
int cell_interval(const sn_record* r, const Cell& c, int32_t kind, int64_t value, int32_t* N) {
  const int64_t slo = bound_ns(r, c, kind, value);
  if (slo < 0) return SN_E_INVAL;
  const int n = sn::min_interval(r->L, c.tc.data(), c.tx.data(), slo);
  if (n < 0 || n > c.n_max) return SN_E_INFEASIBLE;
  *N = n;
  return SN_OK;
}

// ---- a JSON reader for exactly what sn_record_save writes: objects, arrays, integers, strings ----
struct Reader {
  const char* p;
  const char* end;
  bool ok = true;
  void ws() {
    while (p < end && std::isspace((unsigned char)*p)) ++p;
  }
  bool eat(char c) {
    ws();
    if (p < end && *p == c) {
      ++p;
      return true;
    }
    return false;
  }
  bool expect(char c) {
    if (!eat(c)) ok = false;
    return ok;
  }
  std::string str() {
    std::string s;
    if (!expect('"')) return s;
    while (p < end && *p != '"') {
      if (*p == '\\') {   // the writer never escapes; reject
        ok = false;
        return s;
      }
      s.push_back(*p++);
    }
    if (p >= end) ok = false;
    else ++p;
    return s;
  }
  int64_t integer() {
    ws();
    const char* q = p;
    if (q < end && *q == '-') ++q;
    if (q >= end || !std::isdigit((unsigned char)*q)) {
      ok = false;
      return 0;
    }
    char* e = nullptr;
    const long long v = std::strtoll(p, &e, 10);
    if (e == p || e > end || (e < end && (*e == '.' || *e == 'e' || *e == 'E'))) ok = false;
    p = e;
    return (int64_t)v;
  }
  std::vector<int64_t> int_array() {
    std::vector<int64_t> v;
    if (!expect('[')) return v;
    if (eat(']')) return v;
    do v.push_back(integer());
    while (ok && eat(','));
    expect(']');
    return v;
  }
};

}  // namespace

extern "C" int sn_record_create(sn_record** out, int32_t n_layers, int64_t slo_step_ns) {
  if (!out) return SN_E_INVAL;
  *out = nullptr;
  if (n_layers < 1 || slo_step_ns < 0) return SN_E_INVAL;
  sn_record* r = new (std::nothrow) sn_record();
  if (!r) return SN_E_NOMEM;
  r->L = n_layers;
  r->step = slo_step_ns;
  *out = r;
  return SN_OK;
}

extern "C" void sn_record_destroy(sn_record* rec) { delete rec; }
extern "C" int32_t sn_record_layers(const sn_record* rec) { return rec ? rec->L : 0; }
extern "C" int32_t sn_record_cells(const sn_record* rec) { return rec ? (int32_t)rec->cells.size() : 0; }

extern "C" int sn_record_put(sn_record* rec, int32_t phase, int32_t batch, int32_t seq, const int64_t* tc_ns,
                             const int64_t* tx_ns, int32_t n_max) {
  if (!rec || !tc_ns || !tx_ns || bad_phase(phase) || batch < 1 || seq < 1 || n_max < 0 || n_max > rec->L + 1)
    return SN_E_INVAL;
  for (int l = 0; l < rec->L; ++l)
    if (tc_ns[l] < 0 || tx_ns[l] < 0) return SN_E_INVAL;
  Cell c;
  c.tc.assign(tc_ns, tc_ns + rec->L);
  c.tx.assign(tx_ns, tx_ns + rec->L);
  c.n_max = n_max;
  rec->cells[Key{phase, batch, seq}] = std::move(c);
  return SN_OK;
}

extern "C" int sn_record_profile(sn_record* rec, sn_ctx* ctx, int32_t phase, int32_t batch, int32_t seq, int32_t reps) {
  if (!rec || !ctx || bad_phase(phase)) return SN_E_INVAL;
  if (sn_layers(ctx) != rec->L) return SN_E_INVAL;     // the profiler writes one time per context layer
  std::vector<int64_t> tc(rec->L), tx(rec->L);
  const int rc = sn_profile_layers(ctx, phase == SN_PHASE_PREFILL ? 1 : 0, batch, seq, reps, tc.data(), tx.data());
  if (rc != SN_OK) return rc;
  return sn_record_put(rec, phase, batch, seq, tc.data(), tx.data(), sn_max_interval(ctx));
}

extern "C" int sn_record_get(const sn_record* rec, int32_t phase, int32_t batch, int32_t seq, int64_t* tc_ns,
                             int64_t* tx_ns, int32_t* n_max) {
  if (!rec) return SN_E_INVAL;
  const auto it = rec->cells.find(Key{phase, batch, seq});
  if (it == rec->cells.end()) return SN_E_STATE;
  if (tc_ns) std::memcpy(tc_ns, it->second.tc.data(), sizeof(int64_t) * rec->L);
  if (tx_ns) std::memcpy(tx_ns, it->second.tx.data(), sizeof(int64_t) * rec->L);
  if (n_max) *n_max = it->second.n_max;
  return SN_OK;
}

extern "C" int sn_record_cell_interval(const sn_record* rec, int32_t phase, int32_t batch, int32_t seq, int32_t slo_kind,
                                       int64_t slo_value, int32_t* N_out) {
  if (!rec || !N_out) return SN_E_INVAL;
  const auto it = rec->cells.find(Key{phase, batch, seq});
  if (it == rec->cells.end()) return SN_E_STATE;
  return cell_interval(rec, it->second, slo_kind, slo_value, N_out);
}

// The lookup proper; `used`, when given, receives the cells that were consulted.
static int lookup_cells(const sn_record* rec, int32_t phase, int32_t batch, int32_t seq, int32_t slo_kind,
                        int64_t slo_value, int32_t* N_out, std::vector<const Cell*>* used) {
  if (!rec || !N_out || bad_phase(phase) || batch < 1 || seq < 1) return SN_E_INVAL;
  // stored batch sizes and sequence lengths of this phase
  std::set<int32_t> bs, ss;
  for (const auto& kv : rec->cells)
    if (std::get<0>(kv.first) == phase) {
      bs.insert(std::get<1>(kv.first));
      ss.insert(std::get<2>(kv.first));
    }
  auto around = [](const std::set<int32_t>& s, int32_t v, int32_t& lo, int32_t& hi) {
    lo = hi = -1;
    auto it = s.lower_bound(v);            // first >= v
    if (it != s.end()) hi = *it;
    if (it != s.end() && *it == v) lo = v;
    else if (it != s.begin()) lo = *std::prev(it);
  };
  int32_t b_lo, b_hi, s_lo, s_hi;
  around(bs, batch, b_lo, b_hi);
  around(ss, seq, s_lo, s_hi);
  if (b_hi < 0 || s_hi < 0 || !rec->cells.count(Key{phase, b_hi, s_hi})) return SN_E_STATE;
  int32_t best = 0;
  const int32_t cb[2] = {b_lo, b_hi}, cs[2] = {s_lo, s_hi};
  for (int i = 0; i < 2; ++i)
    for (int j = 0; j < 2; ++j) {
      if (cb[i] < 0 || cs[j] < 0) continue;
      const auto it = rec->cells.find(Key{phase, cb[i], cs[j]});
      if (it == rec->cells.end()) continue;
      int32_t n = 0;
      const int rc = cell_interval(rec, it->second, slo_kind, slo_value, &n);
      if (rc != SN_OK) return rc;
      if (n > best) best = n;
      if (used) used->push_back(&it->second);
    }
  *N_out = best;
  return SN_OK;
}

extern "C" int sn_record_lookup(const sn_record* rec, int32_t phase, int32_t batch, int32_t seq, int32_t slo_kind,
                                int64_t slo_value, int32_t* N_out) {
  return lookup_cells(rec, phase, batch, seq, slo_kind, slo_value, N_out, nullptr);
}

extern "C" int sn_record_lookup_refined(const sn_record* rec, int32_t phase, int32_t batch, int32_t seq, int32_t slo_kind,
                                        int64_t slo_value, int32_t* N_out) {
  std::vector<const Cell*> used;
  int32_t n = 0;
  const int rc = lookup_cells(rec, phase, batch, seq, slo_kind, slo_value, &n, &used);
  if (rc != SN_OK) return rc;
  const int L = rec->L;
  *N_out = n;
  if (n > L || used.empty()) return SN_OK;
  // of the intervals that offload as many layers as n, the one whose slowest consulted cell is fastest
  auto worst = [&](int cand) {
    int64_t t = 0;
    for (const Cell* c : used) t = std::max(t, sn::iteration_time(L, c->tc.data(), c->tx.data(), cand, nullptr));
    return t;
  };
  int64_t best_t = worst(n);
  for (int cand = n + 1; cand <= L && sn::offloaded_count(L, cand) == sn::offloaded_count(L, n); ++cand) {
    const int64_t t = worst(cand);
    if (t < best_t) *N_out = cand, best_t = t;
  }
  return SN_OK;
}

extern "C" int sn_record_table(const sn_record* rec, int32_t phase, int32_t slo_kind, int64_t slo_value,
                               const int32_t* batches, int32_t n_batches, const int32_t* seqs, int32_t n_seqs,
                               int32_t* out) {
  if (!rec || !batches || !seqs || !out || n_batches < 0 || n_seqs < 0) return SN_E_INVAL;
  for (int i = 0; i < n_batches; ++i)
    for (int j = 0; j < n_seqs; ++j) {
      int32_t n = 0;
      const int rc = sn_record_lookup(rec, phase, batches[i], seqs[j], slo_kind, slo_value, &n);
      if (rc == SN_OK) out[i * n_seqs + j] = n;
      else if (rc == SN_E_INFEASIBLE) out[i * n_seqs + j] = 0;
      else if (rc == SN_E_STATE) out[i * n_seqs + j] = -1;
      else return rc;
    }
  return SN_OK;
}

extern "C" int sn_record_save(const sn_record* rec, const char* path) {
  if (!rec || !path) return SN_E_INVAL;
  FILE* f = std::fopen(path, "w");
  if (!f) return SN_E_STATE;
  std::fprintf(f, "{\"format\": \"select-n performance record\", \"version\": 1, \"n_layers\": %d, \"slo_step_ns\": %lld, \"cells\": [",
               rec->L, (long long)rec->step);
  bool first = true;
  for (const auto& kv : rec->cells) {
    std::fprintf(f, "%s\n{\"phase\": %d, \"batch\": %d, \"seq\": %d, \"n_max\": %d, \"tc_ns\": [", first ? "" : ",",
                 std::get<0>(kv.first), std::get<1>(kv.first), std::get<2>(kv.first), kv.second.n_max);
    first = false;
    for (int l = 0; l < rec->L; ++l) std::fprintf(f, "%s%lld", l ? ", " : "", (long long)kv.second.tc[l]);
    std::fprintf(f, "], \"tx_ns\": [");
    for (int l = 0; l < rec->L; ++l) std::fprintf(f, "%s%lld", l ? ", " : "", (long long)kv.second.tx[l]);
    std::fprintf(f, "]}");
  }
  std::fprintf(f, "\n]}\n");
  const bool bad = std::ferror(f) != 0;
  return (std::fclose(f) != 0 || bad) ? SN_E_STATE : SN_OK;
}

extern "C" int sn_record_load(sn_record** out, const char* path) {
  if (!out || !path) return SN_E_INVAL;
  *out = nullptr;
  FILE* f = std::fopen(path, "r");
  if (!f) return SN_E_STATE;
  std::string text;
  char buf[1 << 16];
  size_t n;
  while ((n = std::fread(buf, 1, sizeof buf, f)) > 0) text.append(buf, n);
  std::fclose(f);

  Reader rd{text.data(), text.data() + text.size()};
  int64_t L = -1, step = -1, version = -1;
  std::string format;
  struct Raw {
    int64_t phase = -1, batch = -1, seq = -1, n_max = -1;
    std::vector<int64_t> tc, tx;
  };
  std::vector<Raw> raws;
  if (!rd.expect('{')) return SN_E_INVAL;
  if (!rd.eat('}')) {
    do {
      const std::string key = rd.str();
      if (!rd.expect(':')) return SN_E_INVAL;
      if (key == "format") format = rd.str();
      else if (key == "version") version = rd.integer();
      else if (key == "n_layers") L = rd.integer();
      else if (key == "slo_step_ns") step = rd.integer();
      else if (key == "cells") {
        if (!rd.expect('[')) return SN_E_INVAL;
        if (!rd.eat(']')) {
          do {
            Raw c;
            if (!rd.expect('{')) return SN_E_INVAL;
            do {
              const std::string k = rd.str();
              if (!rd.expect(':')) return SN_E_INVAL;
              if (k == "phase") c.phase = rd.integer();
              else if (k == "batch") c.batch = rd.integer();
              else if (k == "seq") c.seq = rd.integer();
              else if (k == "n_max") c.n_max = rd.integer();
              else if (k == "tc_ns") c.tc = rd.int_array();
              else if (k == "tx_ns") c.tx = rd.int_array();
              else return SN_E_INVAL;
            } while (rd.ok && rd.eat(','));
            if (!rd.expect('}')) return SN_E_INVAL;
            raws.push_back(std::move(c));
          } while (rd.ok && rd.eat(','));
          if (!rd.expect(']')) return SN_E_INVAL;
        }
      } else
        return SN_E_INVAL;
    } while (rd.ok && rd.eat(','));
    if (!rd.expect('}')) return SN_E_INVAL;
  }
  rd.ws();
  if (!rd.ok || rd.p != rd.end) return SN_E_INVAL;
  if (format != "select-n performance record" || version != 1 || L < 1 || L > (1 << 20) || step < 0) return SN_E_INVAL;
  sn_record* r = nullptr;
  int rc = sn_record_create(&r, (int32_t)L, step);
  if (rc != SN_OK) return rc;
  for (const Raw& c : raws) {
    if ((int64_t)c.tc.size() != L || (int64_t)c.tx.size() != L || c.phase < 0 || c.phase > 1 || c.batch < 1 ||
        c.batch > INT32_MAX || c.seq < 1 || c.seq > INT32_MAX || c.n_max < 0 || c.n_max > L + 1)
      rc = SN_E_INVAL;
    else
      rc = sn_record_put(r, (int32_t)c.phase, (int32_t)c.batch, (int32_t)c.seq, c.tc.data(), c.tx.data(), (int32_t)c.n_max);
    if (rc != SN_OK) {
      sn_record_destroy(r);
      return rc;
    }
  }
  *out = r;
  return SN_OK;
}
