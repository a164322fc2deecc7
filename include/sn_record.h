/* sn_record.h -- the analyzer's performance record (paper Sec. 4.4, Table 1).
 *
 * For a model on a machine the per-layer compute time depends only on the phase
 * (prefill / decoding) and on the input size (batch size, sequence length), so it is
 * measured once, offline, on a grid of sizes, and the optimal offloading interval of a
 * request is then a table lookup instead of a measurement at serving time.  Prefill and
 * decoding are recorded separately so that each phase gets the interval that suits it
 * (Sec. 4.4, "Supporting the separation of prefill and decoding").
 *
 * A cell (phase, batch, seq) keeps what one profiled iteration measured -- per-layer
 * compute times, per-layer transfer times, the capacity bound on the interval -- rather
 * than one interval per SLO: the interval for ANY latency bound follows exactly from
 * those (the picker of sn.h), and a table like the paper's Table 1 is sn_record_table
 * for one SLO.
 *
 * Conventions as in sn.h: plain C, every function returns SN_OK or a negative SN_E_*
 * code, nothing aborts or throws; all pointers are HOST pointers; one record, one
 * thread.  Pure host code: usable without a GPU, except sn_record_profile.
 */
#ifndef SN_RECORD_H
#define SN_RECORD_H

#include <stdint.h>
#include "sn.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sn_record sn_record;   /* opaque; sn_record_create / _load make it, sn_record_destroy frees it */

enum { SN_PHASE_DECODE = 0, SN_PHASE_PREFILL = 1 };

/* How a latency bound is given:
 *   SN_SLO_ABS_NS        value = the bound in nanoseconds; it is rounded DOWN to the
 *                        record's granularity (the paper's prototype: 2 ms) first.
 *   SN_SLO_REL_PERMILLE  value = the bound as per-mille of the cell's own iteration time
 *                        without offloading: 1500 means 1.5 x, i.e. delta = 0.5 in
 *                        Sec. 4.4's notation.  Integer arithmetic: sum(tc) * value / 1000. */
enum { SN_SLO_ABS_NS = 0, SN_SLO_REL_PERMILLE = 1 };

/* n_layers >= 1; slo_step_ns >= 0 is the granularity of absolute SLOs (0: none). */
int  sn_record_create(sn_record** out, int32_t n_layers, int64_t slo_step_ns);
void sn_record_destroy(sn_record* rec);
int32_t sn_record_layers(const sn_record* rec);      /* 0 for a null record */
int32_t sn_record_cells(const sn_record* rec);       /* number of cells stored */

/* Store (or replace) a cell.  tc_ns, tx_ns: [n_layers] times in ns, all >= 0, copied.
 * n_max: largest interval the GPU's capacity allows for this size (n_layers+1 = no
 * offloading needed to fit; see sn_max_interval). */
int sn_record_put(sn_record* rec, int32_t phase, int32_t batch, int32_t seq, const int64_t* tc_ns,
                  const int64_t* tx_ns, int32_t n_max);

/* The analyzer's measuring step for one size: runs sn_profile_layers(ctx, phase, batch,
 * seq, reps) and stores the result with ctx's capacity bound.  Needs a placed context
 * whose layer count equals the record's; resets the context's KV state (as
 * sn_profile_layers does). */
int sn_record_profile(sn_record* rec, sn_ctx* ctx, int32_t phase, int32_t batch, int32_t seq, int32_t reps);

/* Read a cell back: times copied into tc_ns / tx_ns ([n_layers], either may be NULL),
 * n_max into *n_max (may be NULL).  SN_E_STATE if the cell is not stored. */
int sn_record_get(const sn_record* rec, int32_t phase, int32_t batch, int32_t seq, int64_t* tc_ns,
                  int64_t* tx_ns, int32_t* n_max);

/* Optimal interval of a STORED cell: the smallest N whose iteration meets the bound
 * (n_layers+1: only the un-offloaded iteration does), provided N <= the cell's n_max;
 * SN_E_INFEASIBLE otherwise (reject, Sec. 4.5), SN_E_STATE if the cell is not stored. */
int sn_record_cell_interval(const sn_record* rec, int32_t phase, int32_t batch, int32_t seq, int32_t slo_kind,
                            int64_t slo_value, int32_t* N_out);

/* Interval for ANY size, "conservatively from the nearest combination" (Sec. 4.4): among
 * the batch sizes stored for this phase take the nearest one <= batch and the nearest one
 * >= batch, likewise for sequence lengths; the answer is the LARGEST interval (least
 * offloading) that any of those up to four stored cells asks for.  SN_E_INFEASIBLE if one
 * of them cannot meet the bound; SN_E_STATE if the upper corner (both >=) is not stored,
 * i.e. the query lies beyond the profiled range; lower corners that are not stored are
 * skipped. */
int sn_record_lookup(const sn_record* rec, int32_t phase, int32_t batch, int32_t seq, int32_t slo_kind,
                     int64_t slo_value, int32_t* N_out);

/* sn_record_lookup, then -- keeping the number of host-resident layers floor(n_layers / N) its answer stands for
 * (Sec. 4.3: the same host memory; the paper does not choose between intervals that offload equally many layers)
 * -- the interval whose iteration under Fig. 7's schedule is shortest on the stored times of the cells that were
 * consulted, the slowest of them counting; the smallest such interval on a tie.  Same errors as sn_record_lookup. */
int sn_record_lookup_refined(const sn_record* rec, int32_t phase, int32_t batch, int32_t seq, int32_t slo_kind,
                             int64_t slo_value, int32_t* N_out);

/* A Table-1-like view for one bound: out[i * n_seqs + j] = lookup(batches[i], seqs[j]),
 * 0 where the bound cannot be met, -1 where the record does not cover the size. */
int sn_record_table(const sn_record* rec, int32_t phase, int32_t slo_kind, int64_t slo_value, const int32_t* batches,
                    int32_t n_batches, const int32_t* seqs, int32_t n_seqs, int32_t* out);

/* Persistence: one JSON object {"format", "version", "n_layers", "slo_step_ns", "cells":
 * [{"phase", "batch", "seq", "n_max", "tc_ns": [...], "tx_ns": [...]}, ...]}, cells sorted
 * by (phase, batch, seq).  sn_record_load accepts what sn_record_save writes (any
 * whitespace, any key order); SN_E_INVAL for anything else, SN_E_STATE if the file
 * cannot be opened. */
int sn_record_save(const sn_record* rec, const char* path);
int sn_record_load(sn_record** out, const char* path);

#ifdef __cplusplus
}
#endif
#endif /* SN_RECORD_H */
