/*
 * CPU oracle for post-failure execution-plan scoring (Chameleon, arXiv 2508.21613).
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain, single-threaded definition of
 * what the HIP library computes.  It shares no code, header, table or helper with
 * the HIP path and must never be called from it.  Only tests, the smoke check and
 * the CPU-baseline leg of the benchmark may load it.
 *
 * What each function follows:
 *   - plan tuple (policy, layer distribution, data distribution, failed-node
 *     distribution): Definition 1 ("State") of the Performance Modeling section.
 *   - 1F1B dependency recurrence: Estimator subsection, eq. (transition):
 *     start(i,j) = max(end(i,j-1), end(f1(i), f2(j))) with f1(i)=i-1 for a forward
 *     and i+1 for a backward, f2 = same micro-batch.
 *   - step time of several pipelines = max over pipelines: Estimator subsection,
 *     the equation after eq. (original_step_time).
 *   - data rerouting penalty: eq. (recycle_step_time) and (recycle_step_time_multi).
 *   - batch distribution over pipelines: Planner subsection, "Batch Distribution".
 *   - OOM filter: Planner "Layer Distribution" + Memory Estimator, eq. (peak_memory_decomposed):
 *     peak of the node at position i (0-based) of an n-stage pipeline = static memory of its
 *     layers + (n - i) x activation memory of its layers; with no activation table the peak
 *     is the static sum.
 *   - transition time = restart constant + weight transfer: Estimator subsection,
 *     paragraph on dynamic parallelism; negligible for rerouting.
 *   - which surviving node takes which new stage (transfer_assign = 1): Restorer subsection,
 *     "Weight Transfer": the assignment of least total transfer over the cost matrix
 *     Cost[i][j] = what node i must fetch to become the j-th node of the new pipeline,
 *     by the Kuhn-Munkres algorithm.  The step time keeps the survivors in stage order (the
 *     paper's nodes are identical, so its estimator does not depend on the assignment).
 *   - rounds of gradient communication (allreduce_us > 0): Restorer subsection, "Asymmetric
 *     Communication": greedy colouring of the layer graph whose edges join layers held by one
 *     device; the step time grows by rounds x allreduce_us.  Devices of a plan: redundant
 *     computation - every surviving node holds its stage and its ring successor's; re-partition
 *     - the untouched pipelines' nodes hold the fault-free stages, the j-th survivor of a failed
 *     pipeline holds new stage j; rerouting - every surviving node holds its stage.
 *   - argmin with first-strict-minimum: Algorithm 1, get_execution_plan.
 *
 * Pure conventions with no counterpart in the paper ("parity unpinned": only
 * self-consistency can be tested): plan index order, the fault-free layout P0,
 * the Q16 rounding rule, the redundant-computation load model, the linear cost
 * horizon*t_step + t_trans, and the default constants.
 */
#ifndef CHM_ORACLE_H
#define CHM_ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_OK = 0, ORC_ERR_ARG = -1, ORC_ERR_RANGE = -2, ORC_ERR_OVERFLOW = -3,
       ORC_ERR_UNRECOVERABLE = -4, ORC_ERR_NO_FEASIBLE = -5 };

enum { ORC_MAX_L = 128, ORC_MAX_PP = 32, ORC_MAX_DP = 16, ORC_MAX_M = 256, ORC_MAX_FAILED = 4 };

#define ORC_INF INT64_MAX

typedef struct {
  int32_t L, PP, DP, M;
  const int32_t *fwd_us, *bwd_us, *mem_mib;   /* [L] */
  const uint32_t *speed_q16;                  /* [DP*PP] node id = d*PP+s; NULL = all 65536 */
  int32_t n_failed;
  const int32_t *failed_nodes;                /* [n_failed] */
  int32_t comm_us, mem_cap_mib, reroute_cap, horizon_steps;
  int32_t reconf_us[3];
  int32_t xfer_us_per_mib;
  const int32_t *act_mib;                     /* [L] activation memory per micro-batch in flight; NULL = none */
  int32_t transfer_assign;                    /* re-partition strategy: 0 = the j-th surviving node hosts new stage j,
                                                 1 = the node-to-stage assignment with the least total weight transfer */
  int32_t allreduce_us;                       /* time of one round of data-parallel gradient communication; 0 = not modelled */
} orc_desc;

typedef struct { uint64_t offset, n_part, n_reroute; int32_t stages, strategy; } orc_family;
typedef struct { int32_t n_families; orc_family fam[3]; uint64_t n_plans; } orc_space;

typedef struct {
  uint64_t index; int64_t cost; int32_t strategy, stages;
  uint8_t cuts[32];            /* cuts[0..stages-2] = c_1 < ... < c_k                      */
  int32_t n_affected;          /* affected stages (ascending) for the rerouting family     */
  int32_t affected_stage[4];
  uint16_t reroute[4][16];     /* reroute[a][d] = extra micro-batches on replica d (0 for a failed node) */
  int64_t t_step_us;           /* estimated step time of the plan (0 when it does not fit)  */
  int64_t t_trans_us;          /* its transition time; cost = horizon_steps * t_step_us + t_trans_us */
} orc_plan;

/* --- building blocks, exposed so that tests can pin each one on its own ---------------- */
uint64_t orc_binom(int32_t n, int32_t k);                       /* saturates at UINT64_MAX */
uint64_t orc_partition_rank(int32_t k, const uint8_t *cuts);
void     orc_partition_rank_batch(int32_t k, const uint8_t *cuts, uint64_t n, uint64_t *ranks);  /* cuts[n][k] */
int      orc_partition_unrank(int32_t L, int32_t k, uint64_t rank, uint8_t *cuts);
uint64_t orc_reroute_count(int32_t parts, int32_t total, int32_t cap);
int      orc_reroute_unrank(int32_t parts, int32_t total, int32_t cap, uint64_t rank, uint16_t *r);
uint64_t orc_reroute_rank(int32_t parts, int32_t total, int32_t cap, const uint16_t *r);
int64_t  orc_scale_q16(int64_t x, uint32_t q);
int64_t  orc_makespan_1f1b(int32_t S, const int64_t *F, const int64_t *B, int32_t M);
/* MiB of [a,b) not already held by a node that held [a0,b0); pw = prefix sums of mem, length L+1 */
int64_t  orc_missing_interval(const int64_t *pw, int32_t a, int32_t b, int32_t a0, int32_t b0);
void     orc_distribute_batch(int32_t D, int32_t total, const int32_t *nodes, int32_t *out);
void     orc_layout_p0(int32_t L, int32_t S, int32_t *bounds /* [S+1] */);
/* Minimum total cost of a one-to-one assignment of n nodes to n positions (Restorer, "Weight
 * Transfer": Kuhn-Munkres on the n x n matrix Cost[i][j] = cost for node i to become the j-th
 * node of the new plan).  cost is row-major, cost[i*n+j] >= 0; position_of_node (nullable)
 * receives one optimal assignment. */
int64_t  orc_min_assignment(int32_t n, const int64_t *cost, int32_t *position_of_node);
/* Rounds of data-parallel communication (Restorer, "Asymmetric Communication"): every layer is a
 * vertex, two layers are joined when some device holds both, layers of one colour communicate in
 * the same round.  Greedy colouring: layers in index order, each takes the smallest colour that no
 * already coloured neighbour has; the result is the number of colours used.  holds is row-major
 * [n_devices][L], non-zero where the device holds the layer. */
int32_t  orc_comm_rounds(int32_t L, int32_t n_devices, const uint8_t *holds);

/* --- scenario level ------------------------------------------------------------------- */
typedef struct orc_scenario orc_scenario;
int  orc_open(const orc_desc *d, orc_scenario **out);
void orc_close(orc_scenario *s);
int  orc_plan_space(const orc_scenario *s, orc_space *out);
int  orc_decode(const orc_scenario *s, uint64_t index, orc_plan *out);
/* cost of one explicit plan (no ranking involved): strategy 0/1/2, stage bounds via cuts,
 * reroute[a*16+d] for the rerouting family.  ORC_INF when memory-infeasible. */
int  orc_plan_cost(const orc_scenario *s, int32_t strategy, int32_t k, const uint8_t *cuts,
                   const uint16_t *reroute, int64_t *cost);
int  orc_score(const orc_scenario *s, uint64_t first, uint64_t count, int64_t *costs);
int  orc_score_ranks(const orc_scenario *s, int32_t strategy, const uint64_t *part_ranks,
                     uint64_t n, int64_t *costs);
/* exhaustive argmin; the rerouting family is searched stage by stage (its penalty is a
 * sum of independent per-stage terms), which gives the same answer as the joint sweep. */
int  orc_search(const orc_scenario *s, uint32_t strategy_mask, orc_plan *best);
/* the same over a sub-range of partition ranks of one family (for bounded timing runs);
 * *evals receives the number of (partition, reroute vector) evaluations done. */
int  orc_search_range(const orc_scenario *s, int32_t strategy, uint64_t part_first,
                      uint64_t part_count, orc_plan *best, uint64_t *evals);
/* orc_search_range that also counts, in *fitting, the partitions of the range that pass the memory filter */
int  orc_search_range_counted(const orc_scenario *s, int32_t strategy, uint64_t part_first,
                              uint64_t part_count, orc_plan *best, uint64_t *fitting);
/* plain joint sweep over every index in [first, first+count): slow, for tiny cases */
int  orc_search_joint(const orc_scenario *s, uint64_t first, uint64_t count, orc_plan *best);

/* --- re-planning over DP/PP degrees (Algorithm 1) ---------------------------------------
 * Planner, "Execution Plan Search" and Algorithm 1 (get_parallel_strategy, get_execution_plan),
 * for identical nodes as in the paper.  The surviving nodes are re-laid out as dp pipelines for
 * every dp in [dp_min, dp_max]: integer_partition splits the node count as evenly as possible
 * (the longer pipelines last, as in the paper's 7 nodes -> lengths 2,2,3), a candidate is kept
 * when every length lies in [pp_min, pp_max]; distribute_batch shares the step's micro-batches
 * in proportion to the pipeline lengths; split_layers picks, per pipeline, the contiguous split
 * of the layers with the least 1F1B time among those that fit in memory (here: over ALL
 * C(L-1, n-1) splits, first minimum in rank order; the paper enumerates only the placements of
 * the remainder layers); the step time is the slowest pipeline (+ comm per stage boundary).
 * The transition time is restart + xfer x (least total weight transfer over all one-to-one
 * assignments of the surviving nodes to the positions of the new layout, Kuhn-Munkres).
 * Candidates are ranked by the objective of the "Optimization Problem" paragraph: throughput x
 * effective time ratio = B / t_step x (H - t_trans) / H with H the (constant) time between two
 * faults, compared exactly by cross-multiplication; ties keep the smaller dp. */
typedef struct {
  int32_t L;
  const int32_t *fwd_us, *bwd_us, *mem_mib, *act_mib;   /* [L]; act_mib may be NULL */
  int32_t old_dp, old_pp;                     /* grid before the failure: node d*old_pp+s holds stage s of the even layout */
  int32_t n_failed;
  const int32_t *failed_nodes;
  int32_t dp_min, dp_max, pp_min, pp_max;     /* R_dp, R_pp */
  int32_t micro_batches;                      /* N_m of one step, over all pipelines */
  int32_t comm_us, mem_cap_mib;
  int64_t horizon_us;                         /* H */
  int32_t restart_us, xfer_us_per_mib;
  int32_t allreduce_us;                       /* per communication round, added to the step time after the splits are chosen */
} orc_replan_desc;

typedef struct {
  int32_t found;                              /* 0: no candidate has a layout that fits */
  int32_t n_candidates;                       /* (dp, lengths) pairs that passed the range checks */
  int32_t dp;
  int32_t length[ORC_MAX_DP], micro_batches[ORC_MAX_DP];
  uint8_t cuts[ORC_MAX_DP][32];               /* per pipeline: cuts[0..length-2] */
  int64_t pipeline_us[ORC_MAX_DP];            /* 1F1B time + comm of every pipeline */
  int64_t t_step_us, fetch_mib, t_trans_us;   /* t_step includes comm_rounds x allreduce_us */
  int32_t comm_rounds;
} orc_replan_plan;

/* lengths of dp pipelines over n nodes, as even as possible, the longer ones last; returns 0
 * when dp > n or a length falls outside [pp_min, pp_max] */
int  orc_integer_partition(int32_t n, int32_t dp, int32_t pp_min, int32_t pp_max, int32_t *lengths);
/* best contiguous split of the layers over n stages for a pipeline with M micro-batches
 * (tables as in orc_replan_desc): least orc_makespan_1f1b among the splits whose every stage
 * fits (static + (n - i) x activations <= cap), first minimum in partition-rank order.  Returns
 * ORC_INF when nothing fits. */
int64_t orc_best_split(int32_t L, const int32_t *fwd_us, const int32_t *bwd_us, const int32_t *mem_mib,
                       const int32_t *act_mib, int32_t n, int32_t M, int32_t mem_cap_mib, uint8_t *cuts);
int  orc_replan(const orc_replan_desc *d, orc_replan_plan *out);

#ifdef __cplusplus
}
#endif
#endif
