// Device-side layout of one scenario and the launch interface between the host part
// (chm_host.cpp) and the kernels (chm_kernels.hip).  Internal to libchm.
#ifndef CHM_DEV_H
#define CHM_DEV_H
#include <stdint.h>

#define CHM_INF_COST INT64_MAX
#define CHM_KEY_NONE UINT64_MAX

enum { DEV_MAX_L = 128, DEV_MAX_S = 32, DEV_MAX_D = 16, DEV_MAX_AFF = 4, DEV_MAX_CLS = 16 };

// One distinct pipeline that a plan of a family has to evaluate.  Pipelines of a family
// that are indistinguishable (same nodes' speed factors, same chain, same micro-batch
// count) are merged on the host, so a plan costs one recurrence per class, not per replica.
struct DevClass {
  int32_t n;                    // pipeline length (nodes in the chain)
  int32_t M;                    // micro-batches this pipeline runs
  int32_t pad[2];
  uint8_t src[DEV_MAX_S];       // partition stage whose layers chain position j runs
  uint8_t host[DEV_MAX_S];      // fault-free stage index of the node at chain position j
  uint32_t q[DEV_MAX_S];        // Q16 time multiplier of that node
};

struct DevFamily {
  int32_t strategy;             // 0 redundant, 1 re-partition, 2 rerouting
  int32_t stages;               // stages of the partition (k+1)
  int32_t n_cls;
  int32_t doubled;              // 1: every node also runs its ring successor's stage (strategy 0)
  uint64_t n_part, n_reroute;
  int64_t fixed_step;           // step time of the pipelines the plan does not touch (strategy 1), else 0
  // peak memory of the node(s) running partition stage j = static + mem_coef[j] * activations, where
  // mem_coef[j] is the largest (pipeline length - position) over the pipelines that have such a node
  // (-1: no pipeline has one, the stage is not checked).  For strategy 0 both quantities include the
  // ring successor's stage.
  int32_t mem_coef[DEV_MAX_S];
  DevClass cls[DEV_MAX_CLS];
};

struct DevScenario {
  int32_t L, S, D, M;
  int64_t comm, cap, K, xfer;
  int64_t reconf[3];
  int32_t p0[DEV_MAX_S + 1];    // fault-free layout: stage j = layers [p0[j], p0[j+1])
  int32_t rcap;                 // reroute cap (<=0: none)
  int32_t assign;               // strategy 1: 1 = least-total-transfer assignment of survivors to new stages
  int64_t allreduce;            // time of one round of gradient communication (0: not modelled)
  int32_t p0_max_layers;        // layers of the largest stage of the fault-free layout
  uint32_t node_exists;         // bit s: some pipeline still has its node of stage s (strategy 0's devices)
  int64_t pf[DEV_MAX_L + 1], pb[DEV_MAX_L + 1], pw[DEV_MAX_L + 1];   // prefix sums: forward, backward, static memory
  int64_t pa[DEV_MAX_L + 1];                                          // prefix sums: activation memory
  // rerouting: stages that lost nodes
  int32_t n_aff;
  int32_t aff_stage[DEV_MAX_AFF], aff_peers[DEV_MAX_AFF], aff_total[DEV_MAX_AFF];
  uint32_t aff_q[DEV_MAX_AFF][DEV_MAX_D];      // speed factor of peer i of affected stage a
  uint64_t aff_R[DEV_MAX_AFF];                 // number of valid reroute vectors
  uint32_t comp_off[DEV_MAX_AFF];              // offset of the count table of stage a in comp[]
  uint32_t comp_stride[DEV_MAX_AFF];           // = aff_total[a] + 1
  DevFamily fam[3];                            // indexed by strategy; n_part == 0 when absent
  // strategy 1: the healthy pipelines keep the fault-free layout; their step time does not
  // depend on the plan and is computed once at load into fam[1].fixed_step
  int32_t n_fixed;
  DevClass fixed[DEV_MAX_D];
  // C(x, i) for 0 <= i < DEV_MAX_S, 0 <= x < DEV_MAX_L, saturating
  uint64_t binom[DEV_MAX_S][DEV_MAX_L];
};
// comp[] (separate allocation): for affected stage a, entry [left * stride + rem] is the number
// of valid vectors of `left` entries summing to `rem`.

struct SearchLaunch {
  const DevScenario *scn = nullptr;
  const uint64_t *comp = nullptr;
  int32_t strategy = 0;
  uint64_t part_first = 0;      // first partition rank of this chunk
  uint32_t part_count = 0;      // partitions in this chunk (< 2^idx_bits)
  // A chunk may consist of two windows of ranks: chunk-local index i stands for rank part_first + i, and from
  // i = jump_at on for part_first + i + jump_by (jump_at = ~0: one window).  Lanes then own one partition each.
  uint32_t jump_at = 0xffffffffu;
  uint64_t jump_by = 0;
  int32_t idx_bits = 0;         // low bits of the packed key hold the chunk-local partition index
  // Atomics of many workgroups on one address serialise in the memory system (about 10 ns each), so both
  // targets are spread over slot_mask + 1 words, slot_stride words apart (separate cache lines): workgroup b
  // uses word (b & slot_mask) * slot_stride.  The host takes the minimum / the sum over the words.
  uint64_t *result = nullptr;   // device words, atomicMin target: (cost << idx_bits) | local index
  uint64_t *feasible = nullptr; // device counters: partitions that passed the memory filter (atomicAdd)
  uint32_t slot_mask = 0, slot_stride = 0;
  // list mode: partition i of the chunk is ranks[i] (any order, a rank outside the family counts as
  // infeasible) instead of part_first + i; part_first is then ignored
  const uint64_t *ranks = nullptr;
  // the same with the partitions given by their cut positions: row i = (stages - 1) ascending bytes (a row
  // that is not strictly increasing within 1..L-1 counts as infeasible); at most one of ranks / cuts is set
  const uint8_t *cuts = nullptr;
  // when set, cost i of the chunk (INT64_MAX if infeasible) is also stored to costs_out[i]
  int64_t *costs_out = nullptr;
  // Bounded search (null: every partition that fits is evaluated).  *incumbent = the lowest cost any wave of
  // this search call has evaluated so far (atomicMin, starts at ~0); a partition whose lower bound of the
  // cost lies above it can neither win nor tie and is skipped.  evaluated: counters like `feasible`, of the
  // partitions whose recurrences were run.  Only the specialised range kernels honour it; others evaluate all.
  uint64_t *incumbent = nullptr;
  uint64_t *evaluated = nullptr;
  uint64_t incumbent0 = ~0ull;  // cost of a plan known before the call: what the kernels take *incumbent to be at most
                                // (handed over as an argument, so that the device word needs no fill for it)
};

// End of a search on the device (k_finish_search): which words to combine and where the result record goes.
enum { FINISH_MAX_SLOTS = 16, FINISH_MAX_WAYS = 16 };
// words of the result record
enum { FINISH_COST = 0,        // winner's cost
       FINISH_STRATEGY = 1,    // its strategy, ~0 when nothing fits
       FINISH_PART = 2,        // its partition rank
       FINISH_TRANS = 3,       // its transition time (int64; -1: does not fit, cannot happen for a winner)
       FINISH_RR = 4,          // DEV_MAX_AFF words: rank of its best reroute vector per stage that lost nodes
       FINISH_COUNTS = 8,      // 3 sums of partitions that fit, then 3 sums of partitions evaluated, per strategy
       FINISH_WORDS = 16 };
struct FinishArgs {
  const DevScenario *scn;
  const uint64_t *slots;       // argmin words: slot i owns `ways` words, `stride` words apart, from slots + i * ways * stride
  const uint64_t *counters;    // six counters laid out like six more slots
  uint32_t n_slots, ways, stride;
  int32_t idx_bits;
  int32_t sweep_winner;        // a rerouting winner's best vectors are found here: 1 = by a sweep of one lane per stage that
                               // lost nodes, 2 = from the peers' capacities by one wavefront (spaces too large for one lane), 0 = not
  const uint64_t *comp;        // the reroute count tables (for 2)
  int32_t reset;               // 1: once read, the argmin words go back to "nothing found", the seven counters behind
                               // them (the six summed here and the seeds' own) to 0 and the incumbent word behind those
                               // to "none": the next search with the same layout starts without a fill kernel
  int32_t strategy[FINISH_MAX_SLOTS];
  uint64_t part_first[FINISH_MAX_SLOTS];
  uint32_t jump_at[FINISH_MAX_SLOTS];      // two-window chunks (see SearchLaunch)
  uint64_t jump_by[FINISH_MAX_SLOTS];
  // At most one slot may hold the argmin over an enumerated candidate set of a bounded search: its chunk-local
  // index is a position in cand_cuts (cut positions packed into bytes, 16 bytes per candidate, cand_k of them used),
  // and the candidate's partition rank follows from its cuts.  cand_slot = -1: none.
  int32_t cand_slot, cand_k;
  const void *cand_cuts;
  uint64_t *out;               // FINISH_WORDS words
};
int chmk_finish_search(const FinishArgs &a, int32_t smax, void *stream);

// launch wrappers (defined in chm_kernels.hip); each returns a hipError_t cast to int
int chmk_fixed_pipelines(DevScenario *d_scn, int32_t smax, void *stream);
int chmk_fill_u64(uint64_t *d_ptr, uint32_t n, uint64_t value, void *stream);
// d_ptr[0..zeros) = 0, d_ptr[zeros] = incumbent, d_ptr[key_off .. key_off + keys) = CHM_KEY_NONE (key_off > zeros)
int chmk_init_search(uint64_t *d_ptr, uint32_t zeros, uint64_t incumbent, uint32_t key_off, uint32_t keys, void *stream);
int chmk_score(const DevScenario *d_scn, const uint64_t *d_comp, int32_t strategy, uint64_t first_local,
               uint64_t count, int64_t *d_costs, int32_t smax, void *stream);
int chmk_score_ranks(const DevScenario *d_scn, const uint64_t *d_comp, int32_t strategy,
                     const uint64_t *d_ranks, uint64_t n, int64_t *d_costs, int32_t smax, void *stream);
int chmk_search(const SearchLaunch &a, int32_t smax, void *stream);
int chmk_rank_cuts(const DevScenario *d_scn, int k, const uint8_t *d_cuts, uint64_t n, uint64_t *d_ranks, void *stream);
// writes, per stage that lost nodes, the rank of the best reroute vector of one partition of the rerouting family
// to d_out[0..n_aff): by a sweep of all vectors, or (by_capacity) from the peers' capacities
int chmk_reroute_winner(const DevScenario *d_scn, const uint64_t *d_comp, uint64_t part_rank, int32_t by_capacity,
                        uint64_t *d_out, int32_t smax, void *stream);

// transition time (restart + weight transfer) of one plan into d_out[0], -1 when it does not fit (one lane)
int chmk_plan_transition(const DevScenario *d_scn, int32_t strategy, uint64_t part_rank, int64_t *d_out, int32_t smax,
                         void *stream);
// migration scheme of one pipeline (n survivors, host[i] = fault-free stage of survivor i) for one
// partition of strategy 1: new stage per survivor to d_stage_of_node[0..n), total MiB to *d_fetch_mib
int chmk_transfer_plan(const DevScenario *d_scn, uint64_t part_rank, int32_t n, const uint8_t *host,
                       uint8_t *d_stage_of_node, int64_t *d_fetch_mib, void *stream);

#endif
