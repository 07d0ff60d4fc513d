// Shape-specialised search kernels (chm_fast.hip): interface to the host part.
#ifndef CHM_FAST_H
#define CHM_FAST_H
#include "chm_dev.h"
#include "chm_pool.h"
#include <vector>

enum {
  FAST_MAX_P = 8,            // peers per affected stage the specialised sweeps are instantiated for
  FAST_FUSED_R = 4096,       // up to this many reroute vectors (all stages) the sweep runs inside the search kernel
  FAST_SPLIT_R = 1 << 23,    // up to this many per stage the vectors are tabulated and swept by a kernel of their own
  FAST_SUB = 1 << 20,        // partitions per pass of the split and scoring paths (bounds their scratch memory: 152 MB;
                             // the scratch is sized for the passes actually asked for and grows when needed)
  LIST_SUB = 1 << 24,        // list entries per filter + search pass of explicit lists (scratch: 336 MB when a list is that long)
  LIST_FIRST = 1 << 16       // entries of the first pass of a bounded list search
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
  // and as groups (three or more peers, at most 8 or 16 micro-batches per peer: see k_sweep_groups): all vectors that
  // share their first P-3 entries.  A group is 8 dwords: [0..4] the shared entries, [5] = first value of the entry
  // before the last two, [6] = how many consecutive values it takes, [7] = what the last three entries add up to
  uint32_t grp_off[DEV_MAX_AFF];  // offset (in uint32) of stage a's groups in runs[]
  uint32_t grp_count[DEV_MAX_AFF];
  uint32_t grp_cap[DEV_MAX_AFF];  // 0: stage a has no group table; else the entry limit (8 or 16) its sweep is compiled for
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
  bool mul24_reroute = false;               // peer stage times stay below 2^24: the reroute sweeps may use 24-bit multiplies
  // bounded search on the split path: the least penalty of a stage is found from the peers' capacities
  // (k_least_penalty) instead of sweeping every reroute vector; set by the caller per search
  bool penalty_by_capacity = false;
  // Range search of strategies 0 and 1: share of the partitions that pass the memory filter, estimated at load
  // from FIT_SAMPLES seeded random partitions; below QUEUE_BELOW_SHARE the search compacts the partitions that
  // fit through a ring per wave (k_fast_search, QUEUED).  queue_mode: -1 = by that estimate, 0 = never, 1 = always.
  float fit_share[3] = {1.0f, 1.0f, 1.0f};   // negative: not sampled yet (sampled when a search first asks)
  int queue_mode = -1;
  // Set by the owner of the state before fast_prepare: the stream the library's own uploads and table kernels
  // run on (only that stream is waited for), and a call that waits until no work launched through this handle is
  // in flight any more (made before a buffer that such work may touch is replaced).
  void *load_stream = nullptr;
  PoolStage stage;                          // pinned staging of the uploads at load (the owner's; may be empty)
  void (*quiesce)(void *) = nullptr;
  void *owner = nullptr;
  FastTables h_tables;
  FastTables *d_tables = nullptr;
  uint32_t *d_vecs = nullptr;
  uint32_t *d_runs = nullptr;
  // scratch of the split and scoring paths, FAST_SUB partitions at a time; allocated when first needed
  uint64_t *d_base = nullptr;               // cost without penalties, ~0 for a partition that does not fit
  uint32_t *d_weights = nullptr;            // [partition][affected stage][8] peer stage times
  uint32_t *d_pen = nullptr;                // [partition][4] best penalty per affected stage
  uint64_t *d_rowkey = nullptr;             // [4] (penalty << 32 | row) of the winning partition
  uint32_t *d_fit_list = nullptr;           // [partition] the partitions of the pass that fit in memory, in no particular order
  uint32_t *d_fit_count = nullptr;          // how many of them
  uint32_t scratch_parts = 0;               // partitions d_base, d_weights, d_pen and d_fit_list have room for
  // The run and vector tables of a rerouting family whose vectors are swept by kernels of their own (split) are
  // large (tens of MB, milliseconds to enumerate) and a bounded search never reads them: they are built when an
  // exhaustive search, a cost store or the recovery of a winner's vectors first asks for them.
  bool reroute_tables_ready = false;
  bool vecs_ready = false;                  // the rank-ordered vector table (d_vecs) has been decoded
  size_t vec_words = 0;                     // size of the vector table
  const DevScenario *d_scn = nullptr;       // the handle's device tables (for that later build)
  const uint64_t *d_comp = nullptr;
  // scratch of explicit lists, LIST_SUB entries at a time; allocated when first needed
  void *d_cut_list = nullptr;               // [entry] cut positions of the entries that fit in memory, 16 bytes each
  uint32_t *d_cut_pos = nullptr;            // [entry] their list positions
  uint32_t *d_cut_count = nullptr;          // [workgroup region] how many of its slots are filled
  uint32_t list_capacity = 0;               // entries the three have room for
  // scratch of the candidate path of the bounded search; grown to what a search needs
  void *d_cand_list = nullptr;              // [candidate] cut positions, 16 bytes each
  uint32_t *d_cand_pos = nullptr;           // [candidate] its index
  uint32_t *d_cand_count = nullptr;         // [workgroup] candidates in its region of BLOCK slots
  uint64_t cand_capacity = 0;
  uint64_t *d_cand_ways = nullptr;          // CandidateSet::ways on the device
  uint8_t *d_cand_low = nullptr;            // CandidateSet::low_pair on the device
  size_t cand_ways_capacity = 0;
  uint64_t cand_serial = 0;                 // CandidateSet::serial of the tables the device holds
  uint8_t *h_cand_stage = nullptr;          // pinned staging of the two tables on their way to the device
  size_t cand_stage_capacity = 0;
  void *cand_copied = nullptr;              // hipEvent_t: the last copy out of the staging buffer is done
};

// Bounded search, candidate path.  Every term of the lower bound of a plan's cost belongs to one stage
// (micro-batches x its time + the time of the layers ahead of it, its memory) or, under redundant computation,
// to one node's pair of adjacent stages, and each is monotone in where the stage (or pair) starts: with its end
// fixed, a later start only lowers it.  The partitions whose bound does not exceed the incumbent are therefore
// exactly those whose every stage s starts at or after low_single[s][end] and whose every pair starts at or
// after low_pair[s][end of the pair]: a set that can be counted and enumerated without touching the others.
// ways[s][a][b] = number of ways to place the cuts below a so that stages 0..s obey all of that, stage s being
// layers [a, b).  Candidates are numbered in ascending partition rank (highest cut most significant).
struct CandidateSet {
  int stages = 0, L = 0;
  std::vector<uint64_t> ways;               // [stages][end b][start a], (L+1) x (L+1) per stage; once built, accumulated over
                                            // the starts (entry a = ways with a start <= a), so that a block is found by bisection
  std::vector<uint8_t> low_pair;            // [stages][L+1]: lowest start of the pair (stages s, s+1) that ends at e; 0 = no such limit
  uint64_t total = 0;                       // candidates; 0 also when the bound excludes the whole family
  uint64_t serial = 0;                      // distinguishes the sets a process builds (the device keeps the last one uploaded)
};
enum {
  CAND_DIRECT = 1 << 17,      // up to this many candidates are always enumerated (cheaper than any range search)
  CAND_MAX = 1 << 26,         // and up to this many when the family is too large for a range search,
  CAND_PASS = 1 << 22,        // enumerated and evaluated this many at a time
  CAND_SAMPLE = 1 << 17       // candidates evaluated per round of tightening the incumbent (see run_search)
};

// Counts the candidates of a strategy against an incumbent cost (host).  Returns false when the strategy has no
// specialised kernel, is swept by the split rerouting path, or the tables are out of the candidate path's limits.
bool fast_candidates_build(const FastState *f, const DevScenario &h, int strategy, uint64_t incumbent, CandidateSet *out);
// Enumerates the candidates on the device and runs the search kernel over them; the key written to a.result
// carries the candidate's index.  Same return convention as fast_search.
// Launch index i stands for candidate (a.part_first + i) * stride, a.part_count of them (at most CAND_PASS).
int fast_candidates_search(FastState *f, const DevScenario &h, const SearchLaunch &a, const CandidateSet &cs, uint64_t stride,
                           void *stream);
// Cut positions of candidate `index` (host).
void fast_candidate_cuts(const CandidateSet &cs, uint64_t index, uint8_t *cuts);

// Decides per strategy whether a specialised kernel applies and fills the host copy of its tables (host only;
// a re-partition family whose untouched pipelines do not fit is still reported as covered: its fixed step time
// is only known once the device has computed it).
void fast_select(FastState *f, const DevScenario &h, bool int32_ok);
// fast_select, then uploads the tables.  Returns 0, or non-zero on a failed HIP call.
int fast_prepare(FastState *f, const DevScenario &h, bool int32_ok, const DevScenario *d_scn, const uint64_t *d_comp);
// Launches the specialised search kernel for one chunk.  Returns 0 on success, a positive
// value when the strategy is not covered (the caller then uses the generic kernel), or a
// negative value on a HIP error.
int fast_search(FastState *f, const DevScenario &h, const SearchLaunch &a, void *stream);
// Whether fast_search would run this launch as a bounded search if a.incumbent were set (a range search of a
// covered strategy without cost store whose reroute vectors, if any, are swept inside the search kernel).
bool fast_can_bound(const FastState *f, const SearchLaunch &a);
// Sampled share of partitions of a strategy that pass the memory filter (1.0 where no sample applies).
float fast_fit_share(FastState *f, const DevScenario &h, int strategy);
// Scores plan indices [local_first, local_first+count) of the rerouting family (indices local to
// the family) into d_costs: one pass of the search kernel stores each partition's cost without
// penalties and its peer stage times, then one lane per plan index adds the penalty of its
// reroute vectors (looked up in the rank-ordered table) and stores the cost.  Same return
// convention as fast_search.
int fast_score_reroute(FastState *f, const DevScenario &h, const DevScenario *d_scn, uint64_t local_first,
                       uint64_t count, int64_t *d_costs, void *stream);
// the caller has waited for everything launched through the handle: the buffers can be reused at once
void fast_release(FastState *f);
#endif
