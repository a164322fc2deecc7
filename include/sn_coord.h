/* sn_coord.h -- the per-bus runtime bandwidth coordinator (paper Sec. 4.5, Fig. 8).
 *
 * GPU instances that share a host link each have a minimum offloading interval (below
 * it the request's SLO is violated; it comes from the performance record, sn_record.h)
 * and a maximum interval (above it the model no longer fits the GPU; "infinite" if it
 * fits entirely).  The interval also fixes the link bandwidth an instance consumes.  The
 * coordinator picks, for every instance, an interval within [min, max] such that the
 * consumed bandwidths sum to less than the link's, maximising the host memory in use;
 * each instance then applies its interval with sn_place before its next iteration.
 *
 * Pure host arithmetic (integers only), no GPU needed; conventions as in sn.h.
 */
#ifndef SN_COORD_H
#define SN_COORD_H

#include <stdint.h>
#include "sn.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t  n_layers;       /* L >= 1                                                          */
  int32_t  n_min;          /* smallest interval that meets the SLO, 1..L+1 (L+1: offload
                              nothing)                                                        */
  int32_t  n_max;          /* largest interval capacity allows; >= L+1 means infinite: "no
                              offloading" (interval L+1) is then a legal choice               */
  int32_t  reserved;       /* 0                                                               */
  uint64_t mem_per_layer;  /* bytes moved over the link per offloaded layer per iteration     */
  int64_t  iter_ns;        /* iteration time the consumed bandwidth is computed with, > 0      */
} sn_coord_instance;

#define SN_COORD_MAX_INSTANCES 8

/* Layers offloaded at interval N: floor(L / N) for 1 <= N <= L, else 0. */
int32_t  sn_coord_offloaded(const sn_coord_instance* inst, int32_t N);
/* Host memory in use at interval N: offloaded layers x mem_per_layer. */
uint64_t sn_coord_host_bytes(const sn_coord_instance* inst, int32_t N);
/* Link bandwidth consumed at interval N, bytes per second, rounded down:
 * host_bytes(N) * 1e9 / iter_ns. */
uint64_t sn_coord_rate(const sn_coord_instance* inst, int32_t N);

/* The adjustment of Fig. 8 for n instances (1 <= n <= SN_COORD_MAX_INSTANCES).
 * N_out[n] receives the chosen intervals; host_bytes_out / rate_out (either may be NULL)
 * the totals of the chosen combination.  A combination is valid when every interval lies
 * in [n_min, min(n_max, L+1)] and the rates sum to STRICTLY less than
 * bandwidth_bytes_per_s.  Among the valid ones: most host memory, then least bandwidth,
 * then the lexicographically smallest interval tuple.
 * SN_E_INFEASIBLE: some instance has n_min > n_max (its request cannot be served: return
 * it to the scheduler), or no combination is valid.  SN_E_INVAL: bad arguments. */
int sn_coord_adjust(const sn_coord_instance* inst, int32_t n, uint64_t bandwidth_bytes_per_s, int32_t* N_out,
                    uint64_t* host_bytes_out, uint64_t* rate_out);

#ifdef __cplusplus
}
#endif
#endif /* SN_COORD_H */
