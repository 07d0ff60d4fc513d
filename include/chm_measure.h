/*
 * libchm - measurement, work accounting and tuning.
 *
 * These entry points are no part of the method and of its boundary (include/chm.h): the benchmark and the
 * tests use them to time the kernels of a search with HIP events, to count the work a search did (partitions,
 * reroute vectors, partitions that pass the memory filter: the units the roofline of the kernels is stated in),
 * to measure the VALU issue rates that roofline is checked against, to pick between two kernel variants with
 * equal results, and to ask which kernel family a scenario runs on.  Results of the boundary calls never depend
 * on any of them.
 */
#ifndef CHM_MEASURE_H
#define CHM_MEASURE_H
#include "chm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-call kernel timings (milliseconds between HIP events on the caller's stream),
 * filled by the last chm_search_best on a handle when timing was switched on. */
typedef struct {
  float family_ms[3];          /* main scoring kernel(s) of strategy 0/1/2, 0 when not run           */
  float total_ms;              /* first launch to last launch of the call                            */
  uint64_t partitions[3];      /* partitions evaluated per strategy                                  */
  uint64_t evaluations[3];     /* (partition, reroute vector) evaluations per strategy               */
  uint64_t feasible[3];        /* partitions per strategy that passed the memory filter              */
  uint64_t evaluated[3];       /* of those, partitions whose pipeline recurrences were run: all of
                                * them, or fewer in a bounded search (chm_set_bounded_search)         */
} chm_timing;

/* Which kernels a scenario would run on, decided from the description alone (host only, no device needed; the
 * same decision chm_load_scenario takes).  The estimator's recurrence (eq. (transition)) and its terms are
 * evaluated in int64 by the generic kernels; the shape-specialised kernels evaluate the same integers in int32
 * and are chosen only where load-time bounds show that no intermediate can reach 2^31 (and, for 24-bit
 * multiplies, 2^24), in which case both give the same results.  Tests use this to place scenarios on either
 * side of every such bound. */
typedef struct {
  int32_t idx_bits;              /* low bits of the packed (cost, index) argmin key */
  int32_t int32_recurrence;      /* 1: step time + reroute penalty of every plan stays below 2^31 */
  int32_t present[3];            /* per strategy: it can recover this failure set */
  int32_t specialised[3];        /* per strategy: 1 = the int32 shape-specialised kernels, 0 = the generic int64 ones */
  int32_t sharp_bound[3];        /* per strategy: the bounded search may use its sharper lower bound (24-bit multiplies) */
  int32_t reroute_mul24;         /* peer stage times stay below 2^24 (needed by the specialised rerouting kernels) */
  int32_t reroute_swept_apart;   /* rerouting: more than 4,096 reroute vectors, swept by kernels of their own */
} chm_selection;
int chm_kernel_selection(const chm_scenario_desc *desc, chm_selection *out);

/* Switches event timing of chm_search_best / chm_search_range on or off for a handle,
 * and reads the timings of the last such call. */
int chm_set_timing(chm_scenario *s, int32_t on);
int chm_get_timing(const chm_scenario *s, chm_timing *out);

/* How the range search of the redundant-computation and re-partition strategies treats partitions that fail
 * the memory filter (the OOM filter of the Estimator, "Peak Memory Usage"): mode 1 = every wavefront first
 * collects the partitions that fit and evaluates them 64 at a time with all lanes busy; mode 0 = every lane
 * evaluates its own partitions, lanes whose partition fails idle; mode -1 (the default) = per strategy, mode 1
 * when fewer than 80 % of a seeded sample of partitions fit, else mode 0.  Results do not depend on the mode.
 * share[k] (host, 3 floats, may be NULL) receives the sampled share per strategy (1.0 where no sample was
 * taken).  Errors: CHM_ERR_ARG. */
int chm_set_filter_compaction(chm_scenario *s, int32_t mode, float *share);

/* The distinct pipelines one plan of a strategy has to evaluate (pipelines with the same
 * nodes' speed factors, chain and micro-batch count are merged): *n of them (<= 16), each
 * with length[i] stages and micro_batches[i] micro-batches.  Host only; for work accounting. */
int chm_family_classes(const chm_scenario *s, int32_t strategy, int32_t *n, int32_t *length, int32_t *micro_batches);

/* Shape of the reroute space: *n_affected stages lost nodes; stage a has peers[a] surviving peers
 * and n_vectors[a] valid reroute vectors (arrays of 4).  Host only; for work accounting. */
int chm_reroute_shape(const chm_scenario *s, int32_t *n_affected, int32_t *peers, uint64_t *n_vectors);

/* Measures a VALU integer issue rate of the current device with a register-only kernel and
 * returns executed int32 lane operations per second.  kind 0: independent v_add_u32; kind 1:
 * independent v_max_i32; kind 2: the recurrence cell (v_max_i32 + v_add_u32 in one dependent
 * chain per lane).  iters scales the run time (about 1 ms per 1000).  Synchronises hip_stream.
 * Used by the benchmark to put measured rates beside its nominal roofline peak. */
int chm_valu_probe(int32_t kind, uint32_t iters, double *lane_ops_per_s, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif
