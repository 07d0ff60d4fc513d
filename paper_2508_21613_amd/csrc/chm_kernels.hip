// Generic scoring kernels of libchm for gfx950: any shape within the library limits,
// int64 arithmetic throughout.  One lane evaluates one plan (scoring) or one partition
// with all of its reroute vectors (search).  The shape-specialised kernels live in
// chm_fast.hip and serve searching and scoring alike wherever their load-time bounds hold;
// these are what the library falls back to for every shape and magnitude those do not cover
// (more than 16 stages, times that do not fit int32, more than 8 peers), plus the small
// one-lane kernels around a search (fixed pipelines, the winner's terms, migration scheme).
//
// Pipeline time: the 1F1B dependency recurrence of the Estimator subsection
// (eq. (transition)) is a longest path in a fixed graph, so any topological order gives
// the same integers.  The order used here keeps ONE value per stage live: in round t
// (t = 0 .. M+n-2) stage s runs forward t (if t < M) and then backward t-(n-1-s) (if that
// is a valid micro-batch).  Forward t of stage s needs forward t of stage s-1 (same
// round, swept in stage order) and the stage's previous operation; backward j of stage s
// needs backward j of stage s+1, which stage s+1 ran in round t-1 as its last operation,
// i.e. the value E[s+1] held before this round's forward sweep overwrote it.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <type_traits>

#include "chm_dev.h"

namespace {

constexpr int BLOCK = 256;

__device__ __forceinline__ int64_t imax(int64_t a, int64_t b) { return a > b ? a : b; }
__device__ __forceinline__ int64_t scale_q16(int64_t x, uint32_t q) { return (x * (int64_t)q + 32768) >> 16; }

template <int SMAX>
__device__ __forceinline__ int64_t makespan_generic(const int64_t (&F)[SMAX], const int64_t (&B)[SMAX], int n, int M) {
  int64_t E[SMAX];
#pragma unroll
  for (int s = 0; s < SMAX; ++s) E[s] = 0;
  const int rounds = M + n - 1;
  for (int t = 0; t < rounds; ++t) {
    const bool fwd = t < M;
    int64_t x = 0;
#pragma unroll
    for (int s = 0; s < SMAX; ++s) {
      if (s < n) {
        const int64_t old = E[s];
        if (fwd) {
          E[s] = imax(E[s], x) + F[s];
          x = E[s];
          if (s == n - 1) E[s] += B[s];          // last stage: backward t follows its own forward
        }
        if (s >= 1) {
          const int j = t - n + s;               // micro-batch whose backward stage s-1 runs now
          if (j >= 0 && j < M) E[s - 1] = imax(E[s - 1], old) + B[s - 1];
        }
      }
    }
  }
  return E[0];
}

// cut positions of one lane live in a column of LDS: c[i][tid], i = 0..stages
template <int SMAX>
struct Cuts {
  int32_t (*c)[BLOCK];
  int tid;
  __device__ __forceinline__ int get(int i) const { return c[i][tid]; }
  __device__ __forceinline__ void set(int i, int v) { c[i][tid] = v; }
};

template <int SMAX>
__device__ __forceinline__ void unrank_partition(const DevScenario *scn, int k, uint64_t rank, Cuts<SMAX> cuts) {
  const int L = scn->L;
  cuts.set(0, 0);
  cuts.set(k + 1, L);
  int x = L - 2;
  uint64_t rem = rank;
  for (int i = k; i >= 1; --i) {
    while (scn->binom[i][x] > rem) --x;   // stops at x = i-1 at the latest (C(i-1,i) = 0)
    cuts.set(i, x + 1);
    rem -= scn->binom[i][x];
    --x;
  }
}

__device__ __forceinline__ int64_t missing_interval(const DevScenario *scn, int a, int b, int a0, int b0) {
  const int64_t need = scn->pw[b] - scn->pw[a];
  const int lo = a > a0 ? a : a0, hi = b < b0 ? b : b0;
  const int64_t have = hi > lo ? scn->pw[hi] - scn->pw[lo] : 0;
  return need - have;
}

// Least-transfer assignment of a pipeline's surviving nodes to its new stages (Restorer, "Weight
// Transfer").  A node that takes stage j fetches the stage's layers it does not hold, so the least
// total transfer is the model size minus the largest total overlap of a one-to-one assignment.
// Nodes (by their fault-free stage) and new stages are both in layer order and each side is
// disjoint, so two pairs with a non-zero overlap never cross; pairs without overlap can complete
// any matching.  The optimum is therefore the best non-crossing matching, a two-index recurrence:
// G[i][j] = max(G[i-1][j], G[i][j-1], G[i-1][j-1] + overlap(node i-1, stage j-1)), kept as one row.
template <int SMAX>
__device__ __forceinline__ int64_t best_overlap(const DevScenario *scn, const DevClass &cls, Cuts<SMAX> cuts) {
  int64_t G[SMAX + 1];
#pragma unroll
  for (int j = 0; j <= SMAX; ++j) G[j] = 0;
  for (int i = 0; i < cls.n; ++i) {
    const int lo_i = scn->p0[cls.host[i]], hi_i = scn->p0[cls.host[i] + 1];
    int64_t diag = 0;
#pragma unroll
    for (int j = 0; j < SMAX; ++j) {
      if (j < cls.n) {
        const int a = cuts.get(j), b = cuts.get(j + 1);
        const int lo = a > lo_i ? a : lo_i, hi = b < hi_i ? b : hi_i;
        const int64_t ov = hi > lo ? scn->pw[hi] - scn->pw[lo] : 0;
        const int64_t above = G[j + 1];
        G[j + 1] = imax(imax(above, G[j]), diag + ov);
        diag = above;
      }
    }
  }
  int64_t best = 0;
#pragma unroll
  for (int j = 0; j <= SMAX; ++j) best = (j == cls.n) ? G[j] : best;
  return best;
}

// Rounds of gradient communication of a plan (Restorer, "Asymmetric Communication"): colours the
// greedy colouring in layer order gives the graph that joins layers held by one device.
// Re-partition and rerouting: every device holds one contiguous stage (of the plan's split or of the
// fault-free layout); the layers before l that share a device with l then form one contiguous run
// inside a single stage, all with distinct colours, so l gets a colour below that stage's size and
// the count is the size of the largest stage on any device.
// Redundant computation: a node holds its stage and its ring successor's.  Stage s meets, among the
// stages coloured before it, stage s-1 (through node s-1) and, for the last stage, stage 0 (through
// the last node); its layers take the lowest colours those stages do not use, in order.  Colour sets
// are bit masks (L <= 128 colours).
template <int SMAX>
__device__ __forceinline__ int comm_rounds(const DevScenario *scn, const DevFamily &fam, Cuts<SMAX> cuts) {
  const int SP = fam.stages;
  int rounds = 0;
  if (fam.strategy != 0) {
    for (int j = 0; j < SP; ++j) {
      const int n = cuts.get(j + 1) - cuts.get(j);
      rounds = n > rounds ? n : rounds;
    }
    if (fam.strategy == 1 && scn->n_fixed > 0) rounds = scn->p0_max_layers > rounds ? scn->p0_max_layers : rounds;
    return rounds;
  }
  uint64_t prev_lo = 0, prev_hi = 0, first_lo = 0, first_hi = 0;
  for (int s = 0; s < SP; ++s) {
    const int n = cuts.get(s + 1) - cuts.get(s);
    uint64_t f_lo = 0, f_hi = 0;
    if (s >= 1 && ((scn->node_exists >> (s - 1)) & 1u)) { f_lo |= prev_lo; f_hi |= prev_hi; }
    if (s >= 1 && s == SP - 1 && ((scn->node_exists >> s) & 1u)) { f_lo |= first_lo; f_hi |= first_hi; }
    uint64_t c_lo = 0, c_hi = 0;
    int taken = 0;
    for (int bit = 0; bit < 128 && taken < n; ++bit) {
      const bool used = bit < 64 ? ((f_lo >> bit) & 1ull) : ((f_hi >> (bit - 64)) & 1ull);
      if (used) continue;
      if (bit < 64) c_lo |= 1ull << bit; else c_hi |= 1ull << (bit - 64);
      ++taken;
      rounds = bit + 1 > rounds ? bit + 1 : rounds;
    }
    if (s == 0) { first_lo = c_lo; first_hi = c_hi; }
    prev_lo = c_lo; prev_hi = c_hi;
  }
  return rounds;
}

// Everything of a plan's cost except the rerouting penalty.  Returns false when the plan
// does not fit in memory.
// WITH_TIME = false leaves the pipeline recurrences out (t_step_out is then meaningless): only the memory
// filter and the transition time.
template <int SMAX, bool WITH_TIME = true>
__device__ __forceinline__ bool eval_base(const DevScenario *scn, const DevFamily &fam, Cuts<SMAX> cuts,
                                          int64_t *t_step_out, int64_t *reconf_out) {
  const int SP = fam.stages;
  if (fam.fixed_step == CHM_INF_COST) return false;
  // memory filter
  bool ok = true;
  for (int j = 0; j < SP; ++j) {
    int64_t m = scn->pw[cuts.get(j + 1)] - scn->pw[cuts.get(j)];
    int64_t act = scn->pa[cuts.get(j + 1)] - scn->pa[cuts.get(j)];
    if (fam.doubled) {
      const int nx = (j + 1 == SP) ? 0 : j + 1;
      m += scn->pw[cuts.get(nx + 1)] - scn->pw[cuts.get(nx)];
      act += scn->pa[cuts.get(nx + 1)] - scn->pa[cuts.get(nx)];
    }
    // peak = static + (pipeline length - position) * activations, for the most demanding node of this stage
    const int coef = fam.mem_coef[j];
    ok = ok && (coef < 0 || m + (int64_t)coef * act <= scn->cap);
  }
  if (!ok) return false;

  int64_t t_step = fam.fixed_step;
  int64_t missing = 0;
  if (fam.strategy != 1) {
    for (int j = 0; j < SP; ++j)
      missing += missing_interval(scn, cuts.get(j), cuts.get(j + 1), scn->p0[j], scn->p0[j + 1]);
  }
  for (int ci = 0; ci < fam.n_cls; ++ci) {
    const DevClass &cls = fam.cls[ci];
    int64_t F[SMAX], B[SMAX];
    int64_t miss = 0;
#pragma unroll
    for (int j = 0; j < SMAX; ++j) {
      F[j] = 0; B[j] = 0;
      if (j < cls.n) {
        const int st = cls.src[j];
        const int lo = cuts.get(st), hi = cuts.get(st + 1);
        int64_t f = scn->pf[hi] - scn->pf[lo];
        int64_t b = scn->pb[hi] - scn->pb[lo];
        if (fam.doubled) {
          const int nx = (st + 1 == SP) ? 0 : st + 1;
          const int lo2 = cuts.get(nx), hi2 = cuts.get(nx + 1);
          f += scn->pf[hi2] - scn->pf[lo2];
          b += scn->pb[hi2] - scn->pb[lo2];
        }
        F[j] = scale_q16(f, cls.q[j]);
        B[j] = scale_q16(b, cls.q[j]);
        if (fam.strategy == 1) {
          const int h = cls.host[j];
          miss += missing_interval(scn, lo, hi, scn->p0[h], scn->p0[h + 1]);
        }
      }
    }
    if (fam.strategy == 1 && scn->assign) miss = scn->pw[scn->L] - best_overlap<SMAX>(scn, cls, cuts);
    if (WITH_TIME) {
      const int64_t T = makespan_generic<SMAX>(F, B, cls.n, cls.M) + (int64_t)(cls.n - 1) * scn->comm;
      t_step = imax(t_step, T);
    }
    missing = imax(missing, miss);
  }
  if (WITH_TIME && scn->allreduce > 0) t_step += scn->allreduce * (int64_t)comm_rounds<SMAX>(scn, fam, cuts);
  *t_step_out = t_step;
  *reconf_out = scn->reconf[fam.strategy] + scn->xfer * missing;
  return true;
}

// forward+backward time of affected stage a on its peer i under the lane's partition
template <int SMAX>
__device__ __forceinline__ int64_t peer_weight(const DevScenario *scn, Cuts<SMAX> cuts, int a, int i) {
  const int st = scn->aff_stage[a];
  const int lo = cuts.get(st), hi = cuts.get(st + 1);
  const uint32_t q = scn->aff_q[a][i];
  return scale_q16(scn->pf[hi] - scn->pf[lo], q) + scale_q16(scn->pb[hi] - scn->pb[lo], q);
}

// penalty of the reroute vector of stage a with a given rank (vector decoded on the fly)
template <int SMAX>
__device__ __forceinline__ int64_t penalty_of_rank(const DevScenario *scn, const uint64_t *comp, Cuts<SMAX> cuts,
                                                   int a, uint64_t rank) {
  const int p = scn->aff_peers[a];
  const uint64_t *tab = comp + scn->comp_off[a];
  const uint32_t stride = scn->comp_stride[a];
  int rem = scn->aff_total[a];
  int64_t pen = 0;
  for (int pos = 0; pos < p; ++pos) {
    const int left = p - 1 - pos;
    int v = 0;
    for (;; ++v) {
      const uint64_t cnt = tab[(uint32_t)left * stride + (uint32_t)(rem - v)];
      if (rank < cnt) break;
      rank -= cnt;
    }
    rem -= v;   // a valid rank is always found at a v within [0, min(rem, cap)]
    pen = imax(pen, (int64_t)v * peer_weight<SMAX>(scn, cuts, a, pos));
  }
  return pen;
}

// Sweep of every valid reroute vector of stage a in rank order; first strict minimum.
// The vector lives in a column of LDS.
template <int SMAX>
__device__ __forceinline__ void sweep_stage(const DevScenario *scn, Cuts<SMAX> cuts, int a,
                                            int32_t (*rv)[BLOCK], int64_t *best_pen, uint64_t *best_rank) {
  const int tid = cuts.tid;
  const int p = scn->aff_peers[a];
  const int total = scn->aff_total[a];
  const int cap = scn->rcap > 0 ? scn->rcap : total;
  int64_t w[DEV_MAX_D];
#pragma unroll
  for (int i = 0; i < DEV_MAX_D; ++i) w[i] = i < p ? peer_weight<SMAX>(scn, cuts, a, i) : 0;
  // lexicographically first vector: as much as possible on the last peers
  int rem = total;
  for (int i = p - 1; i >= 0; --i) {
    const int v = rem < cap ? rem : cap;
    rv[i][tid] = v;
    rem -= v;
  }
  int64_t bp = CHM_INF_COST;
  uint64_t br = 0, rank = 0;
  for (;;) {
    int64_t pen = 0;
#pragma unroll
    for (int i = 0; i < DEV_MAX_D; ++i)
      if (i < p) pen = imax(pen, (int64_t)rv[i][tid] * w[i]);
    if (pen < bp) { bp = pen; br = rank; }
    ++rank;
    // successor: rightmost entry that can grow while something to its right can shrink
    int suffix = rv[p - 1][tid];
    int i = p - 2;
    while (i >= 0 && (rv[i][tid] >= cap || suffix == 0)) { suffix += rv[i][tid]; --i; }
    if (i < 0) break;
    rv[i][tid] += 1;
    int left = suffix - 1;
    for (int j = p - 1; j > i; --j) {
      const int v = left < cap ? left : cap;
      rv[j][tid] = v;
      left -= v;
    }
  }
  *best_pen = bp;
  *best_rank = br;
}

// Rank of the best reroute vector of stage a without a sweep, by one wavefront together (all 64 lanes call this
// with the same cuts).  A vector stays within penalty v exactly when every peer i takes at most floor(v / w_i) extra
// micro-batches (w_i = its forward + backward time of the stage), so the least penalty is the least v at which the
// peers' capacities min(cap, floor(v / w_i)) cover the orphans: found by a 64-way search (each lane tries one v per
// round).  Among the vectors within it the lowest rank is the lexicographically smallest one: every peer in turn
// takes as little as the peers after it allow; its rank = the number of valid vectors that are lexicographically
// smaller, read off the count table (the lanes share the additions).  Equals the first minimum of the sweep
// (sweep_stage): same penalty, lowest rank.
template <int SMAX>
__device__ __forceinline__ uint64_t rank_by_capacity(const DevScenario *scn, const uint64_t *comp, Cuts<SMAX> cuts, int a) {
  const int lane = threadIdx.x & 63;
  const int p = scn->aff_peers[a];
  const int64_t orphans = scn->aff_total[a];
  const int64_t cap = scn->rcap > 0 ? scn->rcap : orphans;
  int64_t w[DEV_MAX_D];
  int64_t w_max = 1;
#pragma unroll
  for (int i = 0; i < DEV_MAX_D; ++i) {
    w[i] = i < p ? peer_weight<SMAX>(scn, cuts, a, i) : 0;
    w_max = w[i] > w_max ? w[i] : w_max;
  }
  auto room = [&](int64_t v, int i) -> int64_t {
    const int64_t fit = w[i] == 0 ? cap : v / w[i];
    return fit < cap ? fit : cap;
  };
  auto covers = [&](int64_t v) -> bool {
    int64_t sum = 0;
#pragma unroll
    for (int i = 0; i < DEV_MAX_D; ++i)
      if (i < p) sum += room(v, i);
    return sum >= orphans;
  };
  // least v in [lo, hi] with covers(v); covers(hi) holds (every peer could take all orphans, the cap permitting:
  // the family exists only if the capped peers can absorb them)
  int64_t lo = 0, hi = orphans * w_max;
  while (lo < hi) {                                  // uniform
    const int64_t step = (hi - lo + 62) / 63;          // lane 63 reaches hi
    int64_t mine = lo + (int64_t)lane * step;
    mine = mine < hi ? mine : hi;
    const uint64_t ok = __builtin_amdgcn_ballot_w64(covers(mine));      // lane 63 (or an earlier one) stands at hi
    if (ok == 0) { lo = hi; break; }                 // cannot happen (covers(hi) holds); keeps the loop finite regardless
    const int first = __builtin_ctzll(ok);
    const int64_t at_first = lo + (int64_t)first * step;
    hi = at_first < hi ? at_first : hi;
    lo = first == 0 ? hi : lo + (int64_t)(first - 1) * step + 1;
  }
  const int64_t v = lo;
  const uint64_t *tab = comp + scn->comp_off[a];
  const uint32_t stride = scn->comp_stride[a];
  int64_t rem = orphans;
  uint64_t rank = 0;
  for (int pos = 0; pos < p; ++pos) {                // uniform
    int64_t behind = 0;
#pragma unroll
    for (int i = 0; i < DEV_MAX_D; ++i)
      if (i > pos && i < p) behind += room(v, i);
    const int64_t take = rem - behind > 0 ? rem - behind : 0;
    const uint32_t left = (uint32_t)(p - 1 - pos);
    // vectors whose entry at this position is smaller than `take` (and whose earlier entries agree)
    uint64_t part = 0;
    for (int64_t t = lane; t < take; t += 64) part += tab[left * stride + (uint32_t)(rem - t)];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off, 64);
    rank += part;
    rem -= take;
  }
  return rank;
}

// ---------------------------------------------------------------------------------------
// wave / block argmin on a packed 64-bit key
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t umin64(uint64_t a, uint64_t b) { return a < b ? a : b; }

template <int CTRL>
__device__ __forceinline__ uint64_t dpp_min(uint64_t v) {
  // partner value through a DPP move; lanes without a source keep their own value
  const int lo = __builtin_amdgcn_update_dpp((int)(uint32_t)v, (int)(uint32_t)v, CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp((int)(uint32_t)(v >> 32), (int)(uint32_t)(v >> 32), CTRL, 0xF, 0xF, false);
  return umin64(v, ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

__device__ __forceinline__ uint64_t wave_min(uint64_t v) {
  v = dpp_min<0xB1>(v);     // quad_perm [1,0,3,2]
  v = dpp_min<0x4E>(v);     // quad_perm [2,3,0,1]
  v = dpp_min<0x141>(v);    // row_half_mirror
  v = dpp_min<0x140>(v);    // row_mirror
  // across the four rows of 16 lanes
  v = umin64(v, __shfl_xor(v, 16, 64));
  v = umin64(v, __shfl_xor(v, 32, 64));
  return v;
}

__device__ __forceinline__ void block_min_to_global(uint64_t key, uint64_t *result) {
  __shared__ uint64_t wave_keys[BLOCK / 64];
  key = wave_min(key);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) wave_keys[wave] = key;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint64_t k = wave_keys[0];
#pragma unroll
    for (int i = 1; i < BLOCK / 64; ++i) k = umin64(k, wave_keys[i]);
    if (k != CHM_KEY_NONE) atomicMin((unsigned long long *)result, (unsigned long long)k);
  }
}

// ---------------------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------------------
__global__ void k_fill_u64(uint64_t *p, uint32_t n, uint64_t v) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// start of a search: the `zeros` counter words at the front to 0, the word behind them (the incumbent cost of a bounded
// search) to `incumbent`, and `keys` argmin words from word `key_off` on to "nothing found", in one launch
__global__ void k_init_search(uint64_t *p, uint32_t zeros, uint64_t incumbent, uint32_t key_off, uint32_t keys) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < zeros) p[i] = 0;
  else if (i == zeros) p[i] = incumbent;
  if (i < keys) p[key_off + i] = CHM_KEY_NONE;
}

// step time of the pipelines that strategy 1 leaves in the fault-free layout
template <int SMAX>
__global__ void __launch_bounds__(64) k_fixed_pipelines(DevScenario *scn) {
  // one lane per untouched pipeline (at most DEV_MAX_D <= 64), then the maximum over the wave
  DevFamily &fam = scn->fam[1];
  if (fam.n_part == 0) return;
  const int d = threadIdx.x;
  int64_t t = 0;
  bool fits = true;
  if (d < scn->n_fixed) {
    const DevClass &cls = scn->fixed[d];
    int64_t F[SMAX], B[SMAX];
#pragma unroll
    for (int j = 0; j < SMAX; ++j) {
      F[j] = 0; B[j] = 0;
      if (j < cls.n) {
        const int lo = scn->p0[j], hi = scn->p0[j + 1];
        if (scn->pw[hi] - scn->pw[lo] + (int64_t)(cls.n - j) * (scn->pa[hi] - scn->pa[lo]) > scn->cap) fits = false;
        F[j] = scale_q16(scn->pf[hi] - scn->pf[lo], cls.q[j]);
        B[j] = scale_q16(scn->pb[hi] - scn->pb[lo], cls.q[j]);
      }
    }
    t = makespan_generic<SMAX>(F, B, cls.n, cls.M) + (int64_t)(cls.n - 1) * scn->comm;
  }
  if (!fits) t = CHM_INF_COST;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) t = imax(t, (int64_t)__shfl_xor((long long)t, off, 64));
  if (threadIdx.x == 0) fam.fixed_step = t;
}

template <int SMAX>
__device__ __forceinline__ int64_t plan_cost(const DevScenario *scn, const uint64_t *comp, const DevFamily &fam,
                                             Cuts<SMAX> cuts, uint64_t part_rank, uint64_t rr_rank) {
  unrank_partition<SMAX>(scn, fam.stages - 1, part_rank, cuts);
  int64_t t_step, reconf;
  if (!eval_base<SMAX>(scn, fam, cuts, &t_step, &reconf)) return CHM_INF_COST;
  if (fam.strategy == 2) {
    for (int a = scn->n_aff - 1; a >= 0; --a) {       // last affected stage is least significant
      const uint64_t R = scn->aff_R[a];
      const uint64_t r = rr_rank % R;
      rr_rank /= R;
      t_step += penalty_of_rank<SMAX>(scn, comp, cuts, a, r);
    }
  }
  return scn->K * t_step + reconf;
}

template <int SMAX>
__global__ void __launch_bounds__(BLOCK) k_score(const DevScenario *scn, const uint64_t *comp, int strategy,
                                                 uint64_t first_local, uint64_t count, int64_t *costs) {
  __shared__ int32_t cut_cols[SMAX + 2][BLOCK];
  const uint64_t gid = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
  if (gid >= count) return;
  const DevFamily &fam = scn->fam[strategy];
  Cuts<SMAX> cuts{cut_cols, (int)threadIdx.x};
  const uint64_t local = first_local + gid;
  const uint64_t R = fam.n_reroute;
  const uint64_t part = R == 1 ? local : local / R;
  const uint64_t rr = R == 1 ? 0 : local - part * R;
  costs[gid] = plan_cost<SMAX>(scn, comp, fam, cuts, part, rr);
}

template <int SMAX>
__global__ void __launch_bounds__(BLOCK) k_score_ranks(const DevScenario *scn, const uint64_t *comp, int strategy,
                                                       const uint64_t *ranks, uint64_t n, int64_t *costs) {
  __shared__ int32_t cut_cols[SMAX + 2][BLOCK];
  const uint64_t gid = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
  if (gid >= n) return;
  const DevFamily &fam = scn->fam[strategy];
  Cuts<SMAX> cuts{cut_cols, (int)threadIdx.x};
  const uint64_t part = ranks[gid];
  costs[gid] = part < fam.n_part ? plan_cost<SMAX>(scn, comp, fam, cuts, part, 0) : CHM_INF_COST;
}

template <int SMAX>
__global__ void __launch_bounds__(BLOCK) k_search(SearchLaunch a) {
  __shared__ int32_t cut_cols[SMAX + 2][BLOCK];
  __shared__ int32_t rv_cols[DEV_MAX_D][BLOCK];
  const DevScenario *scn = a.scn;
  const DevFamily &fam = scn->fam[a.strategy];
  const uint32_t gid = blockIdx.x * BLOCK + threadIdx.x;
  uint64_t key = CHM_KEY_NONE;
  bool fits = false;
  if (gid < a.part_count) {
    Cuts<SMAX> cuts{cut_cols, (int)threadIdx.x};
    int64_t t_step = 0, reconf = 0;
    if (a.cuts != nullptr) {
      // explicit cut positions: copy them into the lane's column, checking that they increase within 1..L-1
      const int k = fam.stages - 1;
      const uint8_t *row = a.cuts + (size_t)gid * (size_t)k;
      bool valid = true;
      int prev = 0;
      cuts.set(0, 0);
      cuts.set(k + 1, scn->L);
      for (int i = 1; i <= k; ++i) {
        const int ci = row[i - 1];
        valid = valid && ci > prev && ci <= scn->L - 1;
        cuts.set(i, ci);
        prev = ci;
      }
      if (valid) fits = eval_base<SMAX>(scn, fam, cuts, &t_step, &reconf);
    } else {
      const uint64_t part = a.ranks ? a.ranks[gid] : a.part_first + gid + (gid >= a.jump_at ? a.jump_by : 0);
      if (part < fam.n_part) {
        unrank_partition<SMAX>(scn, fam.stages - 1, part, cuts);
        fits = eval_base<SMAX>(scn, fam, cuts, &t_step, &reconf);
      }
    }
    if (a.costs_out && !fits) a.costs_out[gid] = CHM_INF_COST;
    if (fits) {
      if (fam.strategy == 2) {
        for (int st = 0; st < scn->n_aff; ++st) {
          int64_t pen; uint64_t rk;
          sweep_stage<SMAX>(scn, cuts, st, rv_cols, &pen, &rk);
          t_step += pen;
        }
      }
      const uint64_t cost = (uint64_t)(scn->K * t_step + reconf);
      key = (cost << a.idx_bits) | gid;
      if (a.costs_out) a.costs_out[gid] = (int64_t)cost;
    }
  }
  const uint32_t slot = (blockIdx.x & a.slot_mask) * a.slot_stride;
  const uint64_t n_fit = __popcll(__ballot(fits));
  if ((threadIdx.x & 63) == 0 && n_fit) atomicAdd((unsigned long long *)a.feasible + slot, (unsigned long long)n_fit);
  block_min_to_global(key, a.result + slot);
}

// ranks of the best reroute vectors of ONE partition of the rerouting family (the winner of a search), per stage
// that lost nodes: by a sweep of all vectors (one lane per stage), or, by_capacity, from the peers' capacities
// (one wavefront, stage after stage: for reroute spaces too large to sweep in one lane)
template <int SMAX>
__global__ void __launch_bounds__(BLOCK) k_reroute_winner(const DevScenario *scn, const uint64_t *comp,
                                                          uint64_t part_rank, int by_capacity, uint64_t *out) {
  __shared__ int32_t cut_cols[SMAX + 2][BLOCK];
  __shared__ int32_t rv_cols[DEV_MAX_D][BLOCK];
  const DevFamily &fam = scn->fam[2];
  Cuts<SMAX> cuts{cut_cols, (int)threadIdx.x};
  if (by_capacity) {
    if (threadIdx.x >= 64) return;
    unrank_partition<SMAX>(scn, fam.stages - 1, part_rank, cuts);     // every lane into its own column
    for (int a = 0; a < scn->n_aff; ++a) {
      const uint64_t rk = rank_by_capacity<SMAX>(scn, comp, cuts, a);
      if (threadIdx.x == 0) out[a] = rk;
    }
    return;
  }
  const int a = threadIdx.x;                         // one lane per affected stage
  if (a >= scn->n_aff) return;
  unrank_partition<SMAX>(scn, fam.stages - 1, part_rank, cuts);
  int64_t pen; uint64_t rk;
  sweep_stage<SMAX>(scn, cuts, a, rv_cols, &pen, &rk);
  out[a] = rk;
}

// Migration scheme of one pipeline for one partition of the re-partition strategy: which new stage
// each surviving node hosts and how much it all has to fetch.  One lane; the whole table of the
// non-crossing matching recurrence (see best_overlap) is kept in LDS and walked back from its last
// cell: a step that changes neither index pairs node i-1 with stage j-1.  Nodes left unpaired take
// the stages left over, in ascending order (they hold nothing of them either way).
struct SurvivorList { int32_t n; uint8_t host[DEV_MAX_S]; };

__global__ void __launch_bounds__(64) k_transfer_plan(const DevScenario *scn, uint64_t part_rank, SurvivorList sv,
                                                      uint8_t *stage_of_node, int64_t *fetch_mib) {
  __shared__ int32_t cut_cols[DEV_MAX_S + 2][BLOCK];
  __shared__ int64_t G[DEV_MAX_S + 1][DEV_MAX_S + 1];
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const int n = sv.n;
  Cuts<DEV_MAX_S> cuts{cut_cols, 0};
  unrank_partition<DEV_MAX_S>(scn, n - 1, part_rank, cuts);
  int stage_of[DEV_MAX_S];
  for (int i = 0; i < n; ++i) stage_of[i] = i;
  if (scn->assign) {
    for (int i = 0; i <= n; ++i) { G[i][0] = 0; G[0][i] = 0; }
    for (int i = 1; i <= n; ++i) {
      const int lo_i = scn->p0[sv.host[i - 1]], hi_i = scn->p0[sv.host[i - 1] + 1];
      for (int j = 1; j <= n; ++j) {
        const int a = cuts.get(j - 1), b = cuts.get(j);
        const int lo = a > lo_i ? a : lo_i, hi = b < hi_i ? b : hi_i;
        const int64_t ov = hi > lo ? scn->pw[hi] - scn->pw[lo] : 0;
        G[i][j] = imax(imax(G[i - 1][j], G[i][j - 1]), G[i - 1][j - 1] + ov);
      }
    }
    bool node_done[DEV_MAX_S], stage_taken[DEV_MAX_S];
    for (int i = 0; i < n; ++i) { node_done[i] = false; stage_taken[i] = false; }
    for (int i = n, j = n; i > 0 && j > 0;) {
      if (G[i][j] == G[i - 1][j]) --i;
      else if (G[i][j] == G[i][j - 1]) --j;
      else { stage_of[i - 1] = j - 1; node_done[i - 1] = true; stage_taken[j - 1] = true; --i; --j; }
    }
    int next_free = 0;
    for (int i = 0; i < n; ++i) {
      if (node_done[i]) continue;
      while (stage_taken[next_free]) ++next_free;
      stage_of[i] = next_free;
      stage_taken[next_free] = true;
    }
  }
  int64_t total = 0;
  for (int i = 0; i < n; ++i) {
    const int j = stage_of[i];
    total += missing_interval(scn, cuts.get(j), cuts.get(j + 1), scn->p0[sv.host[i]], scn->p0[sv.host[i] + 1]);
    stage_of_node[i] = (uint8_t)j;
  }
  *fetch_mib = total;
}

// transition time of ONE plan (the winner of a search): out[0] = restart + weight transfer, -1 when the plan
// does not fit.  One lane; no pipeline recurrence (the host takes the step time from cost = horizon x step +
// transition).
template <int SMAX>
__global__ void __launch_bounds__(BLOCK) k_plan_transition(const DevScenario *scn, int strategy, uint64_t part_rank, int64_t *out) {
  __shared__ int32_t cut_cols[SMAX + 2][BLOCK];
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const DevFamily &fam = scn->fam[strategy];
  Cuts<SMAX> cuts{cut_cols, 0};
  unrank_partition<SMAX>(scn, fam.stages - 1, part_rank, cuts);
  int64_t t_step = 0, reconf = 0;
  out[0] = eval_base<SMAX, false>(scn, fam, cuts, &t_step, &reconf) ? reconf : -1;
}

// End of a search on the device: the winner among the argmin words of all launched chunks (lowest cost; among
// equal costs the lowest strategy, then the lowest partition rank: the lowest plan index), the sums of the
// feasibility counters, the winner's transition time and, for data rerouting, the ranks of its best reroute
// vectors, gathered into one record (written straight to pinned host memory when the caller passes such a
// pointer).  One workgroup.  The kernel sits on the critical path of every search, and a single lane chasing
// table entries through global memory pays a microsecond per dependent load, so: all lanes first copy the part of
// the scenario ahead of the binomial table into LDS (SMAX <= 16; the one-lane steps then read LDS), and the
// winner's partition is unranked by the first wavefront together, one table column per digit held across the
// lanes (all columns loaded up front, the digit found with a ballot).
template <int SMAX>
__global__ void __launch_bounds__(BLOCK) k_finish_search(FinishArgs a) {
  constexpr bool STAGED = SMAX <= 16;
  constexpr int HEAD_WORDS = (int)(offsetof(DevScenario, binom) / 8);      // 8-byte words ahead of the binomial table
  __shared__ int32_t cut_cols[SMAX + 2][BLOCK];
  __shared__ int32_t rv_cols[DEV_MAX_D][BLOCK];
  __shared__ uint64_t keys[FINISH_MAX_SLOTS * FINISH_MAX_WAYS];
  __shared__ uint64_t counts[6 * FINISH_MAX_WAYS];
  __shared__ uint64_t win[3];                        // cost, strategy (~0: nothing found), partition rank
  __shared__ uint64_t head[STAGED ? HEAD_WORDS : 1];
  const uint32_t chunk_words = a.ways * a.stride;
  const uint32_t t = threadIdx.x;
  if (t < a.n_slots * a.ways) keys[t] = a.slots[(size_t)(t / a.ways) * chunk_words + (size_t)(t % a.ways) * a.stride];
  if (t < 6 * a.ways) counts[t] = a.counters[(size_t)(t / a.ways) * chunk_words + (size_t)(t % a.ways) * a.stride];
  if (STAGED) {
    const uint64_t *src = (const uint64_t *)a.scn;
    for (int i = (int)t; i < HEAD_WORDS; i += BLOCK) head[i] = src[i];
  }
  if (a.reset) {
    // every word is rewritten by the lane that has just read it (the seventh counter and the incumbent are not read here)
    uint64_t *slots = const_cast<uint64_t *>(a.slots), *counters = const_cast<uint64_t *>(a.counters);
    if (t < a.n_slots * a.ways) slots[(size_t)(t / a.ways) * chunk_words + (size_t)(t % a.ways) * a.stride] = CHM_KEY_NONE;
    if (t < 7 * a.ways) counters[(size_t)(t / a.ways) * chunk_words + (size_t)(t % a.ways) * a.stride] = 0;
    if (t == 0) counters[(size_t)7 * chunk_words] = ~0ull;
  }
  __syncthreads();
  if (t == 0) {
    uint64_t best_cost = ~0ull, best_part = 0;
    int best_strategy = -1;
    for (uint32_t i = 0; i < a.n_slots; ++i) {
      uint64_t key = CHM_KEY_NONE;
      for (uint32_t w = 0; w < a.ways; ++w) key = umin64(key, keys[i * a.ways + w]);
      if (key == CHM_KEY_NONE) continue;
      const uint64_t cost = key >> a.idx_bits;
      const uint64_t local = key & ((1ull << a.idx_bits) - 1ull);
      uint64_t part = a.part_first[i] + local + (local >= a.jump_at[i] ? a.jump_by[i] : 0);
      if ((int)i == a.cand_slot) {
        // a candidate's index: its partition rank = sum of C(c_i - 1, i) over its cut positions
        const uint4 packed = ((const uint4 *)a.cand_cuts)[local];
        const uint32_t words[4] = {packed.x, packed.y, packed.z, packed.w};
        part = 0;
        for (int d = 1; d <= a.cand_k; ++d) {
          const uint32_t cut = (words[(d - 1) >> 2] >> (8 * ((d - 1) & 3))) & 0xffu;
          part += a.scn->binom[d][cut - 1];
        }
      }
      const int strategy = a.strategy[i];
      if (best_strategy < 0 || cost < best_cost ||
          (cost == best_cost && (strategy < best_strategy || (strategy == best_strategy && part < best_part)))) {
        best_cost = cost; best_strategy = strategy; best_part = part;
      }
    }
    win[0] = best_cost; win[1] = best_strategy < 0 ? ~0ull : (uint64_t)best_strategy; win[2] = best_part;
    a.out[FINISH_COST] = best_cost;
    a.out[FINISH_STRATEGY] = win[1];
    a.out[FINISH_PART] = best_part;
    for (int k = 0; k < 6; ++k) {
      uint64_t sum = 0;
      for (uint32_t w = 0; w < a.ways; ++w) sum += counts[k * a.ways + w];
      a.out[FINISH_COUNTS + k] = sum;
    }
  }
  __syncthreads();
  if (win[1] == ~0ull) return;
  const int strategy = (int)win[1];
  const uint64_t part = win[2];
  // what the one-lane steps read: the LDS copy (everything they touch lies ahead of the binomial table), else global
  const DevScenario *scn = STAGED ? (const DevScenario *)head : a.scn;
  const DevFamily &fam = scn->fam[strategy];
  const int k = fam.stages - 1, L = scn->L;
  // ---- unranking by the first wavefront: lane x holds C(x, i) and C(x + 64, i) of every digit i
  if (t < 64) {
    uint64_t rem = part;
    int hi = L - 2;                                  // the digit is the largest x <= hi with C(x, i) <= rem
    for (int i0 = k; i0 >= 1; i0 -= 8) {             // eight digits' columns at a time: their loads are in flight together
      uint64_t lo_col[8], hi_col[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 - u;
        lo_col[u] = i >= 1 ? a.scn->binom[i][t] : 0;
        hi_col[u] = i >= 1 ? a.scn->binom[i][t + 64] : 0;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 - u;
        if (i >= 1) {                                // uniform
          const uint64_t m_hi = __builtin_amdgcn_ballot_w64(hi_col[u] <= rem && (int)t + 64 <= hi);
          const uint64_t m_lo = __builtin_amdgcn_ballot_w64(lo_col[u] <= rem && (int)t <= hi);
          // C(i - 1, i) = 0 <= rem and i - 1 <= hi always: some lane answers
          const int x = m_hi ? 127 - __builtin_clzll(m_hi) : 63 - __builtin_clzll(m_lo);
          const uint64_t taken = m_hi ? __shfl(hi_col[u], x - 64, 64) : __shfl(lo_col[u], x, 64);
          rem -= taken;
          hi = x - 1;
          if (t == 0) { cut_cols[i][0] = x + 1; }
          if (t < DEV_MAX_AFF) cut_cols[i][64 + t] = x + 1;
        }
      }
    }
    if (t == 0) { cut_cols[0][0] = 0; cut_cols[k + 1][0] = L; }
    if (t < DEV_MAX_AFF) { cut_cols[0][64 + t] = 0; cut_cols[k + 1][64 + t] = L; }
  }
  __syncthreads();
  Cuts<SMAX> cuts{cut_cols, (int)t};
  if (t == 0) {
    int64_t t_step = 0, reconf = 0;
    a.out[FINISH_TRANS] = (uint64_t)(eval_base<SMAX, false>(scn, fam, cuts, &t_step, &reconf) ? reconf : (int64_t)-1);
  } else if (a.sweep_winner == 1 && strategy == 2 && t >= 64 && (int)(t - 64) < scn->n_aff) {
    // one lane per stage that lost nodes, in the second wavefront, beside the transition time
    const int st = (int)(t - 64);
    int64_t pen; uint64_t rk;
    sweep_stage<SMAX>(scn, cuts, st, rv_cols, &pen, &rk);
    a.out[FINISH_RR + st] = rk;
  } else if (a.sweep_winner == 2 && strategy == 2 && t >= 64 && t < 128) {
    // reroute spaces too large for one lane: the second wavefront takes the stages one after the other, from
    // the peers' capacities (all its lanes read the cuts of column 64)
    Cuts<SMAX> shared_cuts{cut_cols, 64};
    for (int st = 0; st < scn->n_aff; ++st) {
      const uint64_t rk = rank_by_capacity<SMAX>(scn, a.comp, shared_cuts, st);
      if (t == 64) a.out[FINISH_RR + st] = rk;
    }
  }
}

// partition rank of explicit cut positions (inverse of unrank_partition); cuts[n][k] row-major.
// Cuts that are not strictly increasing within 1..L-1 give UINT64_MAX.
__global__ void __launch_bounds__(BLOCK) k_rank_cuts(const DevScenario *scn, int k, const uint8_t *cuts, uint64_t n,
                                                     uint64_t *ranks) {
  const uint64_t gid = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
  if (gid >= n) return;
  const uint8_t *c = cuts + gid * (uint64_t)k;
  uint64_t r = 0;
  int prev = 0;
  bool valid = true;
  for (int i = 1; i <= k; ++i) {
    const int ci = c[i - 1];
    valid = valid && ci > prev && ci <= scn->L - 1;
    if (valid) r += scn->binom[i][ci - 1];
    prev = ci;
  }
  ranks[gid] = valid ? r : UINT64_MAX;
}

template <typename Fn>
int dispatch_smax(int smax, Fn fn) {
  if (smax <= 4) return fn(std::integral_constant<int, 4>());
  if (smax <= 8) return fn(std::integral_constant<int, 8>());
  if (smax <= 16) return fn(std::integral_constant<int, 16>());
  return fn(std::integral_constant<int, 32>());
}

}  // namespace

int chmk_fill_u64(uint64_t *d_ptr, uint32_t n, uint64_t value, void *stream) {
  hipLaunchKernelGGL(k_fill_u64, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, d_ptr, n, value);
  return (int)hipGetLastError();
}

int chmk_init_search(uint64_t *d_ptr, uint32_t zeros, uint64_t incumbent, uint32_t key_off, uint32_t keys, void *stream) {
  const uint32_t n = (zeros + 1 > keys ? zeros + 1 : keys);
  hipLaunchKernelGGL(k_init_search, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, d_ptr, zeros, incumbent, key_off, keys);
  return (int)hipGetLastError();
}

int chmk_fixed_pipelines(DevScenario *d_scn, int32_t smax, void *stream) {
  return dispatch_smax(smax, [&](auto tag) {
    constexpr int SMAX = decltype(tag)::value;
    hipLaunchKernelGGL(k_fixed_pipelines<SMAX>, dim3(1), dim3(64), 0, (hipStream_t)stream, d_scn);
    return (int)hipGetLastError();
  });
}

int chmk_rank_cuts(const DevScenario *d_scn, int k, const uint8_t *d_cuts, uint64_t n, uint64_t *d_ranks, void *stream) {
  if (n == 0) return 0;
  const uint64_t blocks = (n + BLOCK - 1) / BLOCK;
  if (blocks > 0x7fffffffull) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(k_rank_cuts, dim3((uint32_t)blocks), dim3(BLOCK), 0, (hipStream_t)stream, d_scn, k, d_cuts, n, d_ranks);
  return (int)hipGetLastError();
}

int chmk_score(const DevScenario *d_scn, const uint64_t *d_comp, int32_t strategy, uint64_t first_local,
               uint64_t count, int64_t *d_costs, int32_t smax, void *stream) {
  if (count == 0) return 0;
  const uint64_t blocks = (count + BLOCK - 1) / BLOCK;
  if (blocks > 0x7fffffffull) return (int)hipErrorInvalidValue;
  return dispatch_smax(smax, [&](auto tag) {
    constexpr int SMAX = decltype(tag)::value;
    hipLaunchKernelGGL(k_score<SMAX>, dim3((uint32_t)blocks), dim3(BLOCK), 0, (hipStream_t)stream, d_scn, d_comp,
                       strategy, first_local, count, d_costs);
    return (int)hipGetLastError();
  });
}

int chmk_score_ranks(const DevScenario *d_scn, const uint64_t *d_comp, int32_t strategy, const uint64_t *d_ranks,
                     uint64_t n, int64_t *d_costs, int32_t smax, void *stream) {
  if (n == 0) return 0;
  const uint64_t blocks = (n + BLOCK - 1) / BLOCK;
  if (blocks > 0x7fffffffull) return (int)hipErrorInvalidValue;
  return dispatch_smax(smax, [&](auto tag) {
    constexpr int SMAX = decltype(tag)::value;
    hipLaunchKernelGGL(k_score_ranks<SMAX>, dim3((uint32_t)blocks), dim3(BLOCK), 0, (hipStream_t)stream, d_scn,
                       d_comp, strategy, d_ranks, n, d_costs);
    return (int)hipGetLastError();
  });
}

int chmk_search(const SearchLaunch &a, int32_t smax, void *stream) {
  if (a.part_count == 0) return 0;
  const uint32_t blocks = (a.part_count + BLOCK - 1) / BLOCK;
  return dispatch_smax(smax, [&](auto tag) {
    constexpr int SMAX = decltype(tag)::value;
    hipLaunchKernelGGL(k_search<SMAX>, dim3(blocks), dim3(BLOCK), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
  });
}

int chmk_transfer_plan(const DevScenario *d_scn, uint64_t part_rank, int32_t n, const uint8_t *host,
                       uint8_t *d_stage_of_node, int64_t *d_fetch_mib, void *stream) {
  SurvivorList sv;
  sv.n = n;
  for (int i = 0; i < DEV_MAX_S; ++i) sv.host[i] = i < n ? host[i] : 0;
  hipLaunchKernelGGL(k_transfer_plan, dim3(1), dim3(64), 0, (hipStream_t)stream, d_scn, part_rank, sv, d_stage_of_node,
                     d_fetch_mib);
  return (int)hipGetLastError();
}

int chmk_plan_transition(const DevScenario *d_scn, int32_t strategy, uint64_t part_rank, int64_t *d_out, int32_t smax,
                         void *stream) {
  return dispatch_smax(smax, [&](auto tag) {
    constexpr int SMAX = decltype(tag)::value;
    hipLaunchKernelGGL(k_plan_transition<SMAX>, dim3(1), dim3(BLOCK), 0, (hipStream_t)stream, d_scn, strategy, part_rank, d_out);
    return (int)hipGetLastError();
  });
}

int chmk_finish_search(const FinishArgs &a, int32_t smax, void *stream) {
  if (a.n_slots == 0 || a.n_slots > FINISH_MAX_SLOTS || a.ways == 0 || a.ways > FINISH_MAX_WAYS) return (int)hipErrorInvalidValue;
  return dispatch_smax(smax, [&](auto tag) {
    constexpr int SMAX = decltype(tag)::value;
    hipLaunchKernelGGL(k_finish_search<SMAX>, dim3(1), dim3(BLOCK), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
  });
}

int chmk_reroute_winner(const DevScenario *d_scn, const uint64_t *d_comp, uint64_t part_rank, int32_t by_capacity, uint64_t *d_out,
                        int32_t smax, void *stream) {
  return dispatch_smax(smax, [&](auto tag) {
    constexpr int SMAX = decltype(tag)::value;
    hipLaunchKernelGGL(k_reroute_winner<SMAX>, dim3(1), dim3(BLOCK), 0, (hipStream_t)stream, d_scn, d_comp,
                       part_rank, (int)by_capacity, d_out);
    return (int)hipGetLastError();
  });
}
