// Shape-specialised search kernels (chm_fast.hip): interface to the host part.
#ifndef CHM_FAST_H
#define CHM_FAST_H
#include "chm_dev.h"

enum {
  FAST_MAX_P = 8,            // peers per affected stage the specialised sweeps are instantiated for
  FAST_FUSED_R = 4096,       // up to this many reroute vectors (all stages) the sweep runs inside the search kernel
  FAST_SPLIT_R = 1 << 23,    // up to this many per stage the vectors are tabulated and swept by a kernel of their own
  FAST_SUB = 1 << 18,        // partitions per pass of the split and scoring paths (bounds their scratch memory: 38 MB)
  LIST_SUB = 1 << 22         // list entries per filter + search pass of explicit lists (scratch: 80 MB)
};

// One pipeline class in the form the specialised kernels read (all int32).
struct FastClass {
  int32_t n, M;
  int32_t dead0, dead1;           // partition stages missing from the chain (>= stages: none)
  int32_t unit;                   // 1: every node of the chain runs at nominal speed (no scaling)
  uint32_t q_min;                 // smallest speed factor along the chain (lower bound of the step time)
  int32_t lb_slack;               // what rounding can take from that bound when q_min scales it (0 at nominal speed)
  int32_t comm_total;             // (n-1) * comm
  uint32_t q[DEV_MAX_S];
  int32_t wlo[DEV_MAX_S], whi[DEV_MAX_S];   // memory prefix at the bounds of the fault-free stage of node j
};

struct FastFamily {
  int32_t n_cls;
  int32_t fixed_step;             // strategy 1: step time of the untouched pipelines
  int32_t w0[DEV_MAX_S + 1];      // memory prefix at the fault-free stage bounds
  int32_t w_total;                // memory of the whole model
  int32_t mem_coef[DEV_MAX_S];    // see DevFamily::mem_coef
  int32_t has_act;                // 0: no activation table, the peak is the static sum
  int32_t assign;                 // strategy 1: 1 = least-total-transfer assignment of survivors to new stages
  int32_t allreduce;              // time of one round of gradient communication (0: not modelled)
  int32_t fixed_layers;           // strategy 1: layers of the largest stage on a node of an untouched pipeline, else 0
  uint32_t node_exists;           // strategy 0: bit s = some pipeline still has its node of stage s
  int32_t lb_prefix;              // 1: the sharper lower bound (24-bit multiplies are safe for these times)
  FastClass cls[DEV_MAX_CLS];
};

struct FastTables {
  FastFamily fam[3];
  // rerouting: per affected stage, all valid reroute vectors in rank order; a row has a stride of
  // 4 (up to 4 peers) or 8 dwords, and the row count is padded to a multiple of 4
  uint32_t vec_off[DEV_MAX_AFF];  // offset (in uint32) of stage a's rows in vecs[]
  uint32_t vec_rows[DEV_MAX_AFF]; // rows including the padding
  // the same vectors as runs: all vectors that share their first P-2 entries are consecutive in
  // rank order, the entry before last counts up from `lo` and the last one down.  A run is 8
  // dwords: [0..5] the shared entries, [6] = lo | (sum of the last two entries << 16), [7] = length
  uint32_t run_off[DEV_MAX_AFF];  // offset (in uint32) of stage a's runs in runs[]
  uint32_t run_count[DEV_MAX_AFF];
  // small uncapped reroute spaces have a sweep unrolled at compile time (see sweep_products):
  // peers * 256 + orphaned micro-batches when such a sweep exists for stage a, else 0
  uint32_t unrolled_shape[DEV_MAX_AFF];
  // lower bound of stage a's reroute penalty: some peer takes at least lb_mult[a] = ceil(orphans / peers)
  // micro-batches (0 when a cap below that leaves this unclear), each at a stage time scaled by at least lb_q[a]
  uint32_t lb_mult[DEV_MAX_AFF], lb_q[DEV_MAX_AFF];
};

struct FastState {
  bool usable[3] = {false, false, false};   // per strategy: a specialised kernel covers this scenario
  bool split = false;                       // rerouting: vectors swept by k_sweep instead of inside the search kernel
  // Range search of strategies 0 and 1: share of the partitions that pass the memory filter, estimated at load
  // from FIT_SAMPLES seeded random partitions; below QUEUE_BELOW_SHARE the search compacts the partitions that
  // fit through a ring per wave (k_fast_search, QUEUED).  queue_mode: -1 = by that estimate, 0 = never, 1 = always.
  float fit_share[3] = {1.0f, 1.0f, 1.0f};
  int queue_mode = -1;
  FastTables h_tables;
  FastTables *d_tables = nullptr;
  uint32_t *d_vecs = nullptr;
  uint32_t *d_runs = nullptr;
  // scratch of the split and scoring paths, FAST_SUB partitions at a time; allocated when first needed
  uint64_t *d_base = nullptr;               // cost without penalties, ~0 for a partition that does not fit
  uint32_t *d_weights = nullptr;            // [partition][affected stage][8] peer stage times
  uint32_t *d_pen = nullptr;                // [partition][4] best penalty per affected stage
  uint64_t *d_rowkey = nullptr;             // [4] (penalty << 32 | row) of the winning partition
  // scratch of explicit lists, LIST_SUB entries at a time; allocated when first needed
  void *d_cut_list = nullptr;               // [entry] cut positions of the entries that fit in memory, 16 bytes each
  uint32_t *d_cut_pos = nullptr;            // [entry] their list positions
  uint32_t *d_cut_count = nullptr;          // [workgroup region] how many of its slots are filled
};

// Decides per strategy whether a specialised kernel applies and uploads its tables.
// Returns 0, or non-zero on a failed HIP call.
int fast_prepare(FastState *f, const DevScenario &h, bool int32_ok, const DevScenario *d_scn, const uint64_t *d_comp);
// Launches the specialised search kernel for one chunk.  Returns 0 on success, a positive
// value when the strategy is not covered (the caller then uses the generic kernel), or a
// negative value on a HIP error.
int fast_search(FastState *f, const DevScenario &h, const SearchLaunch &a, void *stream);
// Whether fast_search would run this launch as a bounded search if a.incumbent were set (a range search of a
// covered strategy without cost store whose reroute vectors, if any, are swept inside the search kernel).
bool fast_can_bound(const FastState *f, const SearchLaunch &a);
// Rank of the best reroute vector per affected stage of one partition of the rerouting family,
// written to d_out[0..n_aff).  Same return convention as fast_search.
int fast_reroute_winner(FastState *f, const DevScenario &h, const DevScenario *d_scn, uint64_t part_rank,
                        uint64_t *d_out, void *stream);
// Scores plan indices [local_first, local_first+count) of the rerouting family (indices local to
// the family) into d_costs: one pass of the search kernel stores each partition's cost without
// penalties and its peer stage times, then one lane per plan index adds the penalty of its
// reroute vectors (looked up in the rank-ordered table) and stores the cost.  Same return
// convention as fast_search.
int fast_score_reroute(FastState *f, const DevScenario &h, const DevScenario *d_scn, uint64_t local_first,
                       uint64_t count, int64_t *d_costs, void *stream);
void fast_release(FastState *f);
#endif
