/*
 * libchm - scoring of candidate post-failure execution plans on one AMD MI355X (gfx950).
 *
 * The library implements the hot path behind real-time fault-tolerance policy selection
 * (Chameleon, arXiv 2508.21613): every candidate execution plan - a recovery policy, a
 * contiguous split of the model layers over pipeline stages, and a distribution of the
 * orphaned micro-batches (the execution-plan tuple of Definition 1, "State") - is scored
 * with the step-time estimator of the Estimator subsection (the 1F1B dependency
 * recurrence, eq. (transition); max over pipelines for asymmetric parallelism; the data
 * rerouting terms of eq. (recycle_step_time) / (recycle_step_time_multi)), filtered by
 * the memory estimator, charged a transition time, and the cheapest plan is returned
 * (Algorithm 1, get_execution_plan).  All scoring runs in hand-written HIP kernels: every
 * cost the library returns or stores was computed on the device.  The host side validates,
 * lays out tables, launches, and combines the per-chunk winners when a call has more chunks
 * than the device-side combine takes.  Only a bounded search (chm_set_bounded_search, off by
 * default) does arithmetic of the method on the host, none of it a plan's cost: the ranks of
 * the seed partitions (layer-time and memory quantiles), the per-stage table that counts the
 * partitions whose lower bound stays within the best cost known (fast_candidates_build).
 * There is no CPU fallback: without a usable GPU every compute call returns CHM_ERR_HIP.
 *
 * Conventions
 *   - Every function returns 0 (CHM_OK) or a negative CHM_ERR_* code; nothing throws or
 *     aborts.  chm_strerror() gives a static string for a code.
 *   - Pointers named d_* are DEVICE pointers owned by the caller (allocated with hipMalloc
 *     or, from Python, torch.empty(..., device="cuda").data_ptr()).  All other pointers
 *     are HOST pointers.  Arrays inside chm_scenario_desc are caller-owned and copied by
 *     chm_load_scenario; they may be freed as soon as it returns.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *   - A handle must not be used by two host threads at once; different handles are
 *     independent (loading, searching and freeing one never waits for work of another).  A
 *     handle belongs to the device that was current when it was loaded.  The asynchronous
 *     calls (chm_score_plans, chm_score_ranks, chm_rank_partitions) use scratch of the handle:
 *     a later call on the same handle must be issued on the same stream, or after the caller
 *     has waited for the earlier one.
 *   - Times are int32 microseconds, memory is int32 MiB, speed factors are Q16 time
 *     multipliers (65536 = nominal, 75366 = 15 % slower).  Costs are int64.
 *
 * Plan index space (what a "plan index" means)
 *   Strategies, in this fixed order, each present only if it can recover the failure set:
 *     0  redundant computation   S stages; every node also carries its successor's layers
 *     1  re-partition            the failed pipelines are re-split over their surviving
 *                                nodes (S - failures stages); healthy pipelines keep the
 *                                fault-free layout; micro-batches are redistributed in
 *                                proportion to node counts (Planner, "Batch Distribution")
 *     2  data rerouting          S stages; the failed nodes' micro-batches go to same-stage
 *                                peers of other pipelines
 *   index = family.offset + partition_rank * family.n_reroute + reroute_rank
 *   partition_rank: a split into k+1 non-empty contiguous stages is its set of cut
 *     positions 1 <= c_1 < ... < c_k <= L-1 (stage j = layers [c_j, c_{j+1})); its rank is
 *     sum_i C(c_i - 1, i), the combinatorial number system, in [0, C(L-1, k)).
 *   reroute_rank: for each stage that lost nodes (ascending stage index, first one most
 *     significant) the lexicographic rank, lowest replica most significant, of the vector
 *     of extra micro-batches per surviving peer (entries >= 0, sum = lost nodes * M, each
 *     <= reroute_cap if that is positive).
 *   cost = horizon_steps * t_step + reconf_us[strategy] + xfer_us_per_mib * (MiB of weights
 *     the new layout must fetch); INT64_MAX for a plan whose peak memory exceeds mem_cap_mib on a node.
 */
#ifndef CHM_H
#define CHM_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  CHM_OK = 0,
  CHM_ERR_ARG = -1,            /* null pointer, size out of the limits below, bad node id  */
  CHM_ERR_RANGE = -2,          /* plan range or rank outside the plan space                */
  CHM_ERR_OVERFLOW = -3,       /* plan count or cost bound does not fit 62 bits            */
  CHM_ERR_UNRECOVERABLE = -4,  /* no requested strategy can recover this failure set       */
  CHM_ERR_NO_FEASIBLE = -5,    /* every plan searched exceeds the memory cap               */
  CHM_ERR_HIP = -6,            /* a HIP call failed (no device, launch or copy error)      */
  CHM_ERR_LIMIT = -7           /* chm_search_best_static: the search needs more scratch than its fixed buffer holds */
};

enum { CHM_MAX_L = 128, CHM_MAX_PP = 32, CHM_MAX_DP = 16, CHM_MAX_M = 256, CHM_MAX_FAILED = 4 };

#define CHM_INFEASIBLE INT64_MAX

typedef struct chm_scenario chm_scenario;   /* opaque; owned by the library until chm_free_scenario */

/* Inputs of one failure event: the profiled tables the estimator consumes (System Design,
 * workflow step 1), the DP x PP grid, the micro-batch count and the failed-node set. */
typedef struct {
  int32_t L, PP, DP, M;               /* layers (PP<=L<=128), stages (<=32), pipelines (<=16), micro-batches per pipeline (<=256) */
  const int32_t *fwd_us, *bwd_us;     /* [L] per-layer forward / backward time, each >= 1            */
  const int32_t *mem_mib;             /* [L] per-layer memory, each >= 0                             */
  const uint32_t *speed_q16;          /* [DP*PP] node id = d*PP+s, in [1, 2^20]; NULL = all 65536    */
  int32_t n_failed;                   /* 0..4                                                        */
  const int32_t *failed_nodes;        /* [n_failed] distinct node ids                                */
  int32_t comm_us;                    /* added once per stage boundary of a pipeline, >= 0           */
  int32_t mem_cap_mib;                /* per-node memory limit, >= 1                                 */
  int32_t reroute_cap;                /* max extra micro-batches per peer; <= 0 = no cap             */
  int32_t horizon_steps;              /* training steps until the next failure is expected, >= 1     */
  int32_t reconf_us[3];               /* per-strategy restart constant, >= 0                         */
  int32_t xfer_us_per_mib;            /* weight-transfer cost rate, >= 0                             */
  const int32_t *act_mib;             /* [L] activation memory per micro-batch in flight, each >= 0; NULL = none.
                                         With it mem_mib is the static part (weights, optimizer states, gradients) and
                                         the node at position i (from 0) of an n-stage pipeline peaks at
                                         static + (n - i) * activations (Memory Estimator, eq. peak_memory_decomposed) */
  int32_t transfer_assign;            /* re-partition strategy, which surviving node hosts which new stage when the weights
                                         to fetch are counted: 0 = the j-th survivor (in stage order) hosts new stage j;
                                         1 = the one-to-one assignment with the least total transfer (Restorer, "Weight
                                         Transfer": minimum-cost matching on Cost[i][j] = MiB node i must fetch to hold new
                                         stage j).  The step time keeps the survivors in stage order in both cases. */
  int32_t allreduce_us;               /* time of one round of data-parallel gradient communication, >= 0; 0 = not modelled.
                                         The step time of a plan grows by rounds x allreduce_us, rounds = colours the greedy
                                         colouring (layers in index order, smallest free colour) gives the graph whose vertices
                                         are the layers and whose edges join layers held by one device (Restorer, "Asymmetric
                                         Communication").  Devices: redundant computation - every surviving node holds its
                                         stage and its ring successor's; re-partition - nodes of untouched pipelines hold the
                                         fault-free stages, the j-th survivor of a failed pipeline holds new stage j;
                                         rerouting - every surviving node holds its stage. */
} chm_scenario_desc;

typedef struct { uint64_t offset, n_part, n_reroute; int32_t stages, strategy; } chm_family;
typedef struct { int32_t n_families; chm_family fam[3]; uint64_t n_plans; } chm_space;

typedef struct {
  uint64_t index;              /* global plan index; UINT64_MAX when nothing feasible was found      */
  int64_t cost;                /* CHM_INFEASIBLE when nothing feasible was found                      */
  int32_t strategy, stages;
  uint8_t cuts[32];            /* cuts[0..stages-2] = c_1 < ... < c_k                                 */
  int32_t n_affected;          /* rerouting only: stages that lost nodes, ascending                   */
  int32_t affected_stage[4];
  uint16_t reroute[4][16];     /* reroute[a][d] = extra micro-batches on pipeline d for affected stage a */
  int64_t t_step_us;           /* estimated step time of the plan (Estimator), 0 when nothing feasible was found or
                                  the plan was only decoded                                               */
  int64_t t_trans_us;          /* its transition time; cost = horizon_steps * t_step_us + t_trans_us      */
} chm_best;

/* Validates the description, builds the plan space and uploads the scenario tables
 * (Definition 1; Algorithm 1 inputs).  Synchronous.  Errors: CHM_ERR_ARG, CHM_ERR_OVERFLOW,
 * CHM_ERR_HIP.  On error *out is NULL. */
int chm_load_scenario(const chm_scenario_desc *desc, chm_scenario **out);

/* The families present for this failure set and the number of plan indices. Host only. */
int chm_plan_space(const chm_scenario *s, chm_space *out);

/* Scores plan indices [first, first+count) into d_costs[0..count) (device, int64).
 * Asynchronous on hip_stream.  Errors: CHM_ERR_ARG, CHM_ERR_RANGE, CHM_ERR_HIP. */
int chm_score_plans(chm_scenario *s, uint64_t first, uint64_t count, int64_t *d_costs, void *hip_stream);

/* Scores n explicit partitions of one strategy, given by their partition ranks in device
 * memory, with reroute rank 0 (the strategy must have n_reroute == 1, else CHM_ERR_ARG).
 * A rank outside the family gives cost CHM_INFEASIBLE for that entry.  Asynchronous. */
int chm_score_ranks(chm_scenario *s, int32_t strategy, const uint64_t *d_part_ranks, uint64_t n,
                    int64_t *d_costs, void *hip_stream);

/* Partition ranks of n explicit partitions of one strategy: d_cuts (device, uint8) holds n rows of
 * (stages-1) cut positions c_1 < ... < c_k; d_part_ranks (device) receives the ranks, UINT64_MAX
 * for a row that is not strictly increasing within 1..L-1.  Asynchronous on hip_stream. */
int chm_rank_partitions(chm_scenario *s, int32_t strategy, const uint8_t *d_cuts, uint64_t n,
                        uint64_t *d_part_ranks, void *hip_stream);

/* Argmin over n explicit partitions of one strategy (partition ranks in device memory): each
 * partition is scored as in chm_search_best (for data rerouting with every reroute vector).
 * *position (nullable) receives the first list position that holds the minimum, d_costs
 * (nullable, device) the cost of every list entry (CHM_INFEASIBLE for a partition that does
 * not fit or a rank outside the family).  Synchronises hip_stream.  Errors as chm_search_best. */
int chm_search_ranks(chm_scenario *s, int32_t strategy, const uint64_t *d_part_ranks, uint64_t n,
                     int64_t *d_costs, chm_best *out, uint64_t *position, void *hip_stream);

/* The same for partitions given by their cut positions: d_cuts (device, uint8) holds n rows of
 * (stages-1) ascending cut positions, as for chm_rank_partitions; a malformed row counts as a partition
 * that does not fit.  Skips the ranking and unranking of the list, which dominates for deep pipelines. */
int chm_search_cuts(chm_scenario *s, int32_t strategy, const uint8_t *d_cuts, uint64_t n,
                    int64_t *d_costs, chm_best *out, uint64_t *position, void *hip_stream);

/* Exhaustive argmin over the strategies in strategy_mask (bit k = strategy k): every
 * partition of every selected family is scored on the device; for data rerouting every
 * reroute vector of every stage that lost nodes is scored (the penalty is a sum of
 * independent per-stage terms, so stages are swept one after the other).  Ties go to the
 * lowest plan index.  Synchronises hip_stream before returning.  Errors:
 * CHM_ERR_UNRECOVERABLE (mask selects no existing family), CHM_ERR_NO_FEASIBLE (out is
 * filled with index UINT64_MAX, cost CHM_INFEASIBLE), CHM_ERR_OVERFLOW (the selected families hold more
 * than 2^16 chunks of 2^idx_bits partitions, idx_bits <= 30: beyond exhaustive reach; search windows with
 * chm_search_range or lists instead), CHM_ERR_ARG, CHM_ERR_HIP. */
int chm_search_best(chm_scenario *s, uint32_t strategy_mask, chm_best *out, void *hip_stream);

/* chm_search_best on n distinct handles of one device in one call (the plan cache of the Planner's overhead
 * paragraph: the best plan for every failure set that may occur, searched ahead of time).  The searches of all
 * handles are launched back to back and the host waits once for the whole batch instead of once per handle.
 * From 8 handles on they are dealt out over four streams of the library's own (default priority), which start
 * behind the work already queued on hip_stream and which hip_stream waits for before the call returns, so that
 * the kernels of different handles overlap at their ends; timings read with chm_get_timing then include that
 * overlap.  outs[i] and codes[i] (host arrays of n) receive what chm_search_best would have returned for
 * handles[i], bounded or exhaustive as set on each handle.  Returns CHM_OK when every search ran (codes[i] may
 * still be CHM_ERR_NO_FEASIBLE, CHM_ERR_UNRECOVERABLE, CHM_ERR_OVERFLOW), CHM_ERR_ARG for a null or repeated
 * handle or handles of different devices, CHM_ERR_HIP when a HIP call failed.  Synchronises hip_stream. */
int chm_search_best_batch(chm_scenario *const *handles, int32_t n, uint32_t strategy_mask, chm_best *outs,
                          int32_t *codes, void *hip_stream);

/* chm_search_best for callers that cannot allocate device memory while they run (code under HIP graph capture
 * around it, tight serving loops, harnesses that forbid hipMalloc): the same exhaustive search with the same
 * result, but every device word the call needs beyond the handle's tables - the per-chunk argmin words, the
 * feasibility counters, the winner's reroute ranks and transition time - lives in one fixed device array of
 * 65,664 bytes inside the library (one copy per GPU, held until the process ends) instead of buffers taken
 * from the allocator.  The call makes no hipMalloc, hipFree or other allocating call.  Always exhaustive
 * (chm_set_bounded_search is ignored).  Limits: at most 8,184 chunks of 2^idx_bits partitions (CHM_ERR_LIMIT
 * beyond; with the usual idx_bits of 30 that is every space chm_search_best accepts short of 2^43 partitions),
 * and no rerouting family whose reroute vectors are swept by kernels of their own (more than 4,096 vectors
 * over its stages: CHM_ERR_LIMIT, use chm_search_best).  On CHM_ERR_LIMIT out is filled as for
 * CHM_ERR_NO_FEASIBLE.  All calls on one GPU share the array, which keeps the last call's contents (the
 * call resets what it reads): two calls that overlap in time on one GPU, from any handles or threads, race.
 * Otherwise as chm_search_best (synchronises hip_stream; same errors). */
int chm_search_best_static(chm_scenario *s, uint32_t strategy_mask, chm_best *out, void *hip_stream);

/* The same over partition ranks [part_first, part_first+part_count) of one strategy. */
int chm_search_range(chm_scenario *s, int32_t strategy, uint64_t part_first, uint64_t part_count,
                     chm_best *out, void *hip_stream);

/* Migration scheme of one plan of the re-partition strategy (Restorer, "Weight Transfer"): for the
 * partition with rank part_rank and pipeline `pipeline` (one that lost nodes), *n_nodes = its
 * surviving nodes, node_stage[i] = fault-free stage of the i-th of them (ascending), stage_of_node[i]
 * = the new stage that node hosts, *fetch_mib = MiB of weights the nodes fetch in total (the figure
 * the plan's cost charges, maximised over the pipelines that lost nodes).  With transfer_assign = 1
 * this is an assignment of least total transfer (one of them when several tie), with 0 the survivors
 * in stage order.  Arrays of 32 bytes each, host memory.  The scheme is computed on the device;
 * synchronises hip_stream.  Errors: CHM_ERR_UNRECOVERABLE (the strategy does not exist for this
 * failure set), CHM_ERR_ARG (pipeline out of range or intact), CHM_ERR_RANGE, CHM_ERR_HIP. */
int chm_transfer_plan(chm_scenario *s, uint64_t part_rank, int32_t pipeline, int32_t *n_nodes,
                      uint8_t *node_stage, uint8_t *stage_of_node, int64_t *fetch_mib, void *hip_stream);

/* Host-only structural decoding of a plan index (cost is not evaluated and is set to 0). */
int chm_decode_plan(const chm_scenario *s, uint64_t index, chm_best *out);

/* Bounded search, off by default.  on = 1 (on = 2: the same with the size thresholds below set to one
 * partition, so that tests reach every path on small scenarios): chm_search_best and chm_search_range skip a partition as soon as a
 * lower bound of its cost (micro-batches x the largest forward + backward time of a stage, which every
 * pipeline needs under the dependencies of eq. (transition); plus lower bounds of the communication rounds
 * and of the reroute penalty of eq. (re-route); the transition time counted as its constant part) lies
 * above the lowest cost evaluated so far in the same call.  The plan returned is the same, ties included:
 * only plans that can neither win nor tie are skipped, one by one or a run of consecutive ranks at a time
 * (the stages above the cuts that change within the run are common to all of its partitions, and so is their
 * share of the bound), or never enumerated at all: for a family searched as a whole the library counts on
 * the host, stage by stage, the partitions whose bound stays within the best cost known, and the device
 * enumerates and evaluates only those (this also reaches families of more than 2^46 partitions, which
 * chm_search_best otherwise refuses with CHM_ERR_OVERFLOW, whenever at most 2^26 candidates remain).  The search
 * starts with the ranks around the time-balanced and the memory-balanced partition of each range, so that a
 * good cost is known early.  chm_timing.evaluated (chm_measure.h) tells how many
 * partitions were evaluated in full; chm_timing.feasible then counts only those partitions that were looked
 * at one by one and fit.  Where the reroute vectors of a stage are too many to sweep inside the search kernel,
 * a bounded search finds the least penalty of eq. (re-route) from the peers' capacities instead of sweeping them
 * (some vector stays within v exactly when the peers can take all orphaned micro-batches within v each).  Covers
 * the range and list searches of the specialised kernels without cost store (other paths evaluate everything;
 * with a cost store every cost is wanted and nothing is skipped).  Errors: CHM_ERR_ARG. */
int chm_set_bounded_search(chm_scenario *s, int32_t on);

/* ---- Re-planning over DP/PP degrees (Planner, "Execution Plan Search" and Algorithm 1) --------------
 * Identical nodes, as in the paper.  The nodes that survive are re-laid out as dp pipelines for every dp
 * in [dp_min, dp_max]: the node count is split as evenly as possible (integer_partition; the longer
 * pipelines last, 7 nodes over 3 pipelines = 2,2,3), a candidate is kept when every pipeline length lies
 * in [pp_min, pp_max]; the step's micro-batches are shared in proportion to the lengths (distribute_batch);
 * for every pipeline ALL contiguous splits of the layers over its stages are scored on the device (1F1B
 * recurrence, memory filter) and the first minimum in partition-rank order is taken (split_layers; the
 * paper enumerates only the placements of the remainder layers); the step time is the slowest pipeline,
 * with comm_us per stage boundary.  Transition time = restart_us + xfer_us_per_mib x the least total MiB
 * the nodes must fetch over all one-to-one assignments of surviving nodes to positions of the new layout
 * (Restorer, "Weight Transfer"; solved on the device).  Candidates are ranked by the objective of the
 * "Optimization Problem" paragraph, throughput x effective time ratio = B / t_step x (H - t_trans) / H,
 * compared exactly; ties keep the smaller dp. */
typedef struct {
  int32_t L;                                  /* layers, 1..128 */
  const int32_t *fwd_us, *bwd_us, *mem_mib;   /* [L], host; as in chm_scenario_desc */
  const int32_t *act_mib;                     /* [L] or NULL */
  int32_t old_dp, old_pp;                     /* grid before the failure: node d*old_pp+s holds stage s of the even layout */
  int32_t n_failed;                           /* 0 .. old_dp*old_pp */
  const int32_t *failed_nodes;                /* [n_failed] distinct node ids */
  int32_t dp_min, dp_max;                     /* R_dp, within 1..16 */
  int32_t pp_min, pp_max;                     /* R_pp, within 1..32 */
  int32_t micro_batches;                      /* N_m of one step over all pipelines, >= 1; a pipeline runs at most 256: a dp
                                                 whose batch distribution would give some pipeline more is not a candidate */
  int32_t comm_us, mem_cap_mib;
  int64_t horizon_us;                         /* H: time between two faults (transition + training), >= 1 */
  int32_t restart_us, xfer_us_per_mib;
  int32_t allreduce_us;                       /* per round of gradient communication (see chm_scenario_desc), added to the
                                                 step time of a candidate after its splits are chosen; 0 = not modelled */
  int32_t bounded_search;                     /* != 0: the split searches skip splits whose lower bound of the pipeline
                                                 time lies above the best one found (chm_set_bounded_search); same plan */
} chm_replan_desc;

typedef struct {
  int32_t found;                              /* 0: no candidate in range has a layout that fits in memory */
  int32_t n_candidates;                       /* (dp, lengths) pairs that passed the range checks */
  int32_t dp;
  int32_t length[16], micro_batches[16];      /* per pipeline of the chosen plan */
  uint8_t cuts[16][32];                       /* per pipeline: cuts[0..length-2] */
  int64_t pipeline_us[16];                    /* 1F1B time + comm of every pipeline */
  int64_t t_step_us, fetch_mib, t_trans_us;   /* t_step_us includes comm_rounds x allreduce_us */
  int32_t comm_rounds;                        /* 0 when allreduce_us is 0 */
  /* work accounting of the call (all candidates, not only the chosen one) */
  uint64_t splits_scored;                     /* contiguous splits scored by the search kernels */
  uint64_t splits_feasible;                   /* of which passed the memory filter (bounded: of those looked at one by one) */
  uint64_t splits_evaluated;                  /* of which had their recurrence run (all of them unless bounded_search) */
  double algorithmic_ops;                     /* 4n per split + (4nM + 6n + 4) per split that fits, n stages, M micro-batches */
  float search_ms, assign_ms;                 /* HIP-event time of the split-search kernels / of the assignment kernels */
} chm_replan_plan;

/* Runs the search above.  All pointers are host pointers; tables are copied.  Synchronises hip_stream.
 * Errors: CHM_ERR_ARG, CHM_ERR_OVERFLOW (a split space or cost bound beyond 62 bits), CHM_ERR_HIP.
 * No candidate / nothing fits is not an error: CHM_OK with out->found = 0. */
int chm_replan(const chm_replan_desc *desc, chm_replan_plan *out, void *hip_stream);

/* The re-plans for the loss of 1 .. k nodes (Planner, overhead paragraph: the optimal plans for potential failure
 * scenarios are computed ahead of time and looked up when a fault occurs; Algorithm 1, get_parallel_strategy: the
 * loop over failure counts).  desc->failed_nodes gives the order in which the nodes are taken to fail; plans[i-1]
 * (host array of k, k <= desc->n_failed) receives what chm_replan returns when the first i of them have failed.
 * The best split of the layers over a pipeline of given length and micro-batch count is searched once for the whole
 * table, so an entry's work accounting (splits_scored ...) covers only the searches no earlier entry has made.
 * Errors as chm_replan; synchronises hip_stream. */
int chm_replan_table(const chm_replan_desc *desc, int32_t k, chm_replan_plan *plans, void *hip_stream);

/* Ranks two plans by the objective of the "Optimization Problem" paragraph, throughput x effective time
 * ratio = B / t_step x (H - t_trans) / H for the same global batch B and time H between two faults: returns
 * 1 when plan a is better, -1 when plan b is better, 0 on an exact tie (compared by cross-multiplication in
 * 128 bits).  Lets a caller choose between the winner of chm_search_best (recovery inside the DP x PP grid)
 * and that of chm_replan (new DP/PP degrees) from their t_step_us / t_trans_us.  Host only.  Step times
 * must be positive; CHM_ERR_ARG (-1 is a valid answer, so errors are reported as -100) otherwise. */
int chm_compare_objective(int64_t t_step_a_us, int64_t t_trans_a_us, int64_t t_step_b_us, int64_t t_trans_b_us,
                          int64_t horizon_us);

void chm_free_scenario(chm_scenario *s);
const char *chm_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif
