// Re-planning over DP/PP degrees (Planner, Algorithm 1) on top of the split-search kernels, and the
// device solver for the least-transfer assignment of surviving nodes to the positions of a new
// layout (Restorer, "Weight Transfer").
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <map>
#include <utility>
#include <vector>

#include "chm_internal.h"
#include "chm_pool.h"

// typed front ends of the caching allocator (chm_pool.h)
template <typename T>
static inline bool pool_take(T *&p, size_t bytes) { p = (T *)pool_device_alloc(bytes); return p != nullptr; }
template <typename T>
static inline bool pool_take_pinned(T *&p, size_t bytes) { p = (T *)pool_pinned_alloc(bytes); return p != nullptr; }

namespace {

enum { RP_MAX_NODES = CHM_MAX_DP * CHM_MAX_PP, RP_MAX_L = CHM_MAX_L };

struct AssignArgs {
  int32_t n;                                   // nodes = positions
  int32_t L;
  const int32_t *held;                         // [2n] device: layers [lo, hi) every node holds
  const int32_t *pos;                          // [2n] device: layers [lo, hi) of every position
  const int64_t *pw;                           // [L+1] device: prefix sums of per-layer memory
  int64_t *total;                              // device: least total MiB
  int32_t *position_of_node;                   // [n] device: one optimal assignment
  int32_t *rounds;                             // device: layers of the largest position = rounds of gradient communication
};

// Minimum-cost one-to-one assignment (Kuhn-Munkres with potentials), one wavefront.  Rows (nodes)
// are inserted one at a time; for the new row the cheapest augmenting path is grown over reduced
// costs cost - u[row] - v[col]: every step scans all columns outside the tree (lanes take columns
// 64 apart), the column with the least slack joins (wave minimum of slack << 10 | column, so ties
// take the lowest column), potentials move by that slack, until a free column is reached; then the
// matching is flipped along the path.  Cost[i][j] is never stored: it is the memory of position
// j's layers minus what node i already holds of them, two prefix-sum reads.
__global__ void __launch_bounds__(64) k_min_assignment(AssignArgs a) {
  __shared__ int64_t pw[RP_MAX_L + 1];
  __shared__ int64_t u[RP_MAX_NODES + 1], v[RP_MAX_NODES + 1], slack[RP_MAX_NODES + 1];
  __shared__ int32_t row_of_col[RP_MAX_NODES + 1], prev_col[RP_MAX_NODES + 1];
  __shared__ int32_t h_lo[RP_MAX_NODES], h_hi[RP_MAX_NODES], p_lo[RP_MAX_NODES + 1], p_hi[RP_MAX_NODES + 1];
  __shared__ uint8_t in_tree[RP_MAX_NODES + 1];
  __shared__ uint64_t pick;
  const int n = a.n, lane = threadIdx.x;
  const int64_t BIG = INT64_MAX / 4;
  for (int i = lane; i <= a.L; i += 64) pw[i] = a.pw[i];
  for (int i = lane; i < n; i += 64) {
    h_lo[i] = a.held[2 * i]; h_hi[i] = a.held[2 * i + 1];
    p_lo[i] = a.pos[2 * i]; p_hi[i] = a.pos[2 * i + 1];
    u[i] = 0;
  }
  for (int c = lane; c <= n; c += 64) { v[c] = 0; row_of_col[c] = -1; }
  __syncthreads();
  for (int r = 0; r < n; ++r) {
    for (int c = lane; c <= n; c += 64) { slack[c] = BIG; prev_col[c] = n; in_tree[c] = 0; }
    if (lane == 0) row_of_col[n] = r;           // column n: virtual start column of the new row
    __syncthreads();
    int c0 = n;
    for (;;) {
      if (lane == 0) in_tree[c0] = 1;
      __syncthreads();
      const int r0 = row_of_col[c0];
      const int hl = h_lo[r0], hh = h_hi[r0];
      const int64_t u0 = u[r0];
      uint64_t key = ~0ull;
      for (int c = lane; c < n; c += 64) {
        if (in_tree[c]) continue;
        const int lo = p_lo[c] > hl ? p_lo[c] : hl, hi = p_hi[c] < hh ? p_hi[c] : hh;
        const int64_t cost = pw[p_hi[c]] - pw[p_lo[c]] - (hi > lo ? pw[hi] - pw[lo] : 0);
        const int64_t red = cost - u0 - v[c];
        if (red < slack[c]) { slack[c] = red; prev_col[c] = c0; }
        const uint64_t k = ((uint64_t)slack[c] << 10) | (uint64_t)c;     // slack >= 0 and below 2^53
        key = k < key ? k : key;
      }
      for (int off = 32; off > 0; off >>= 1) {
        const uint64_t other = __shfl_xor(key, off, 64);
        key = other < key ? other : key;
      }
      if (lane == 0) pick = key;
      __syncthreads();
      const int64_t step = (int64_t)(pick >> 10);
      const int c_next = (int)(pick & 1023u);
      for (int c = lane; c <= n; c += 64) {
        if (in_tree[c]) { u[row_of_col[c]] += step; v[c] -= step; }     // tree columns hold distinct rows
        else slack[c] -= step;
      }
      __syncthreads();
      c0 = c_next;
      if (row_of_col[c0] < 0) break;            // a free column: augment
    }
    if (lane == 0) {
      while (c0 != n) {
        const int pc = prev_col[c0];
        row_of_col[c0] = row_of_col[pc];
        c0 = pc;
      }
    }
    __syncthreads();
  }
  int64_t part = 0;
  for (int c = lane; c < n; c += 64) {
    const int i = row_of_col[c];
    const int lo = p_lo[c] > h_lo[i] ? p_lo[c] : h_lo[i], hi = p_hi[c] < h_hi[i] ? p_hi[c] : h_hi[i];
    part += pw[p_hi[c]] - pw[p_lo[c]] - (hi > lo ? pw[hi] - pw[lo] : 0);
    a.position_of_node[i] = c;
  }
  // every position holds one contiguous range of layers, so the greedy colouring of the layer graph
  // (Restorer, "Asymmetric Communication") needs exactly as many rounds as the largest position has layers
  int most = 0;
  for (int c = lane; c < n; c += 64) most = p_hi[c] - p_lo[c] > most ? p_hi[c] - p_lo[c] : most;
  for (int off = 32; off > 0; off >>= 1) {
    part += __shfl_xor(part, off, 64);
    const int other = __shfl_xor(most, off, 64);
    most = other > most ? other : most;
  }
  if (lane == 0) { *a.total = part; *a.rounds = most; }
}

struct Scratch {
  int32_t *d_held = nullptr, *d_pos = nullptr, *d_assign = nullptr;
  int64_t *d_pw = nullptr, *d_total = nullptr; // d_total: [0] least total MiB, [1] rounds (int32 in its low half)
  int64_t *h_total = nullptr;                  // pinned, two words
  hipStream_t stream = nullptr;                // the stream every kernel and copy that touches these blocks runs on
  ~Scratch() {
    (void)hipStreamSynchronize(stream);        // (an early return may leave work in flight)
    if (d_held) pool_release(d_held);
    if (d_pos) pool_release(d_pos);
    if (d_assign) pool_release(d_assign);
    if (d_pw) pool_release(d_pw);
    if (d_total) pool_release(d_total);
    if (h_total) pool_release(h_total);
  }
};

struct SplitResult { int rc; int64_t cost; uint8_t cuts[32]; };

struct Events {
  hipEvent_t a = nullptr, b = nullptr;
  bool ok() { return hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess; }
  ~Events() { if (a) (void)hipEventDestroy(a); if (b) (void)hipEventDestroy(b); }
};

int check(const chm_replan_desc *d) {
  if (!d) return CHM_ERR_ARG;
  if (d->L < 1 || d->L > CHM_MAX_L || !d->fwd_us || !d->bwd_us || !d->mem_mib) return CHM_ERR_ARG;
  if (d->old_dp < 1 || d->old_dp > CHM_MAX_DP || d->old_pp < 1 || d->old_pp > CHM_MAX_PP || d->old_pp > d->L) return CHM_ERR_ARG;
  if (d->n_failed < 0 || d->n_failed > d->old_dp * d->old_pp || (d->n_failed > 0 && !d->failed_nodes)) return CHM_ERR_ARG;
  if (d->dp_min < 1 || d->dp_max < d->dp_min || d->dp_max > CHM_MAX_DP) return CHM_ERR_ARG;
  if (d->pp_min < 1 || d->pp_max < d->pp_min || d->pp_max > CHM_MAX_PP) return CHM_ERR_ARG;
  if (d->micro_batches < 1 || d->comm_us < 0 || d->mem_cap_mib < 1 || d->horizon_us < 1 || d->restart_us < 0 ||
      d->xfer_us_per_mib < 0 || d->allreduce_us < 0)
    return CHM_ERR_ARG;
  for (int l = 0; l < d->L; ++l)
    if (d->fwd_us[l] < 1 || d->bwd_us[l] < 1 || d->mem_mib[l] < 0 || (d->act_mib && d->act_mib[l] < 0)) return CHM_ERR_ARG;
  return CHM_OK;
}

}  // namespace

extern "C" int chm_compare_objective(int64_t t_step_a_us, int64_t t_trans_a_us, int64_t t_step_b_us, int64_t t_trans_b_us,
                                     int64_t horizon_us) {
  if (t_step_a_us < 1 || t_step_b_us < 1 || horizon_us < 1) return -100;
  // (H - trans_a) / step_a  versus  (H - trans_b) / step_b
  const __int128 lhs = ((__int128)horizon_us - t_trans_a_us) * t_step_b_us;
  const __int128 rhs = ((__int128)horizon_us - t_trans_b_us) * t_step_a_us;
  return lhs > rhs ? 1 : (lhs < rhs ? -1 : 0);
}

namespace {
typedef std::map<std::pair<int, int>, SplitResult> SplitCache;   // (stages, micro-batches) -> best split of the layers
int replan_core(const chm_replan_desc *d, chm_replan_plan *out, void *hip_stream, SplitCache &best_split);
}  // namespace

extern "C" int chm_replan(const chm_replan_desc *d, chm_replan_plan *out, void *hip_stream) {
  SplitCache cache;
  return replan_core(d, out, hip_stream, cache);
}

extern "C" int chm_replan_table(const chm_replan_desc *d, int32_t k, chm_replan_plan *plans, void *hip_stream) {
  if (!d || !plans || k < 0 || k > d->n_failed) return CHM_ERR_ARG;
  // The tables, ranges and limits are the same for every entry, so the best split of the layers over a pipeline
  // of given length and micro-batch count is searched once for the whole table.
  SplitCache cache;
  for (int32_t i = 1; i <= k; ++i) {
    chm_replan_desc di = *d;
    di.n_failed = i;
    const int rc = replan_core(&di, &plans[i - 1], hip_stream, cache);
    if (rc) return rc;
  }
  return CHM_OK;
}

namespace {
int replan_core(const chm_replan_desc *d, chm_replan_plan *out, void *hip_stream, SplitCache &best_split) {
  if (!out) return CHM_ERR_ARG;
  memset(out, 0, sizeof(*out));
  int rc = check(d);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  const int L = d->L, old_nodes = d->old_dp * d->old_pp;
  std::vector<char> dead(old_nodes, 0);
  for (int i = 0; i < d->n_failed; ++i) {
    const int n = d->failed_nodes[i];
    if (n < 0 || n >= old_nodes || dead[n]) return CHM_ERR_ARG;
    dead[n] = 1;
  }
  // what every surviving node holds: its stage of the even layout (extra layers on the last stages)
  std::vector<int> p0(d->old_pp + 1, 0);
  for (int s = 0; s < d->old_pp; ++s) p0[s + 1] = p0[s] + L / d->old_pp + (s >= d->old_pp - L % d->old_pp ? 1 : 0);
  std::vector<int32_t> held;
  for (int n = 0; n < old_nodes; ++n)
    if (!dead[n]) { held.push_back(p0[n % d->old_pp]); held.push_back(p0[n % d->old_pp + 1]); }
  const int N = (int)held.size() / 2;
  std::vector<int64_t> pw(L + 1, 0);
  for (int l = 0; l < L; ++l) pw[l + 1] = pw[l] + d->mem_mib[l];
  // the transition time must stay far from the int64 range
  if ((unsigned __int128)d->xfer_us_per_mib * (unsigned __int128)pw[L] * (unsigned)(N > 0 ? N : 1) + (unsigned)d->restart_us >=
      ((unsigned __int128)1 << 62))
    return CHM_ERR_OVERFLOW;

  Scratch sc;
  sc.stream = st;
  if (N > 0) {
    bool ok = pool_take(sc.d_held, held.size() * sizeof(int32_t));
    ok = ok && pool_take(sc.d_pos, held.size() * sizeof(int32_t));
    ok = ok && pool_take(sc.d_assign, (size_t)N * sizeof(int32_t));
    ok = ok && pool_take(sc.d_pw, pw.size() * sizeof(int64_t));
    ok = ok && pool_take(sc.d_total, 2 * sizeof(int64_t));
    ok = ok && pool_take_pinned(sc.h_total, 2 * sizeof(int64_t));
    ok = ok && hipMemcpyAsync(sc.d_held, held.data(), held.size() * sizeof(int32_t), hipMemcpyHostToDevice, st) == hipSuccess;
    ok = ok && hipMemcpyAsync(sc.d_pw, pw.data(), pw.size() * sizeof(int64_t), hipMemcpyHostToDevice, st) == hipSuccess;
    ok = ok && hipStreamSynchronize(st) == hipSuccess;
    if (!ok) return CHM_ERR_HIP;
  }

  Events ev;
  if (!ev.ok()) return CHM_ERR_HIP;
  uint64_t splits_scored = 0, splits_feasible = 0, splits_evaluated = 0;
  double algorithmic_ops = 0;
  float search_ms = 0, assign_ms = 0;
  bool have = false;
  __int128 best_gain = 0;
  int64_t best_step = 1;
  for (int dp = d->dp_min; dp <= d->dp_max; ++dp) {
    if (dp > N) break;
    int len[CHM_MAX_DP], mb[CHM_MAX_DP];
    bool in_range = d->micro_batches >= dp;
    for (int p = 0; p < dp; ++p) {
      len[p] = N / dp + (p >= dp - N % dp ? 1 : 0);
      in_range = in_range && len[p] >= d->pp_min && len[p] <= d->pp_max && len[p] <= L;
    }
    if (!in_range) continue;
    chm_internal_share_micro_batches(dp, d->micro_batches, len, mb);
    // a pipeline runs at most CHM_MAX_M micro-batches: a layout that would give one more is not a candidate
    bool share_ok = true;
    for (int p = 0; p < dp; ++p) share_ok = share_ok && mb[p] <= CHM_MAX_M;
    if (!share_ok) continue;
    ++out->n_candidates;
    chm_replan_plan cand;
    memset(&cand, 0, sizeof(cand));
    cand.dp = dp;
    bool fits = true;
    for (int p = 0; p < dp && fits; ++p) {
      const std::pair<int, int> key(len[p], mb[p]);
      auto it = best_split.find(key);
      if (it == best_split.end()) {
        SplitResult r;
        memset(&r, 0, sizeof(r));
        chm_scenario *pipe = nullptr;
        r.rc = chm_internal_load_pipeline(L, d->fwd_us, d->bwd_us, d->mem_mib, d->act_mib, len[p], mb[p], d->comm_us,
                                          d->mem_cap_mib, &pipe);
        if (r.rc) return r.rc;
        chm_best b;
        chm_timing tm;
        (void)chm_set_timing(pipe, 1);
        (void)chm_set_bounded_search(pipe, d->bounded_search);
        r.rc = chm_search_best(pipe, 1u << 1, &b, hip_stream);
        (void)chm_get_timing(pipe, &tm);
        chm_free_scenario(pipe);
        splits_scored += tm.partitions[1];
        splits_feasible += tm.feasible[1];
        splits_evaluated += tm.evaluated[1];
        search_ms += tm.family_ms[1];
        algorithmic_ops += 4.0 * len[p] * (double)tm.partitions[1] +
                           (4.0 * len[p] * mb[p] + 6.0 * len[p] + 4.0) * (double)tm.feasible[1];
        if (r.rc != CHM_OK && r.rc != CHM_ERR_NO_FEASIBLE) return r.rc;
        r.cost = b.cost;
        memcpy(r.cuts, b.cuts, sizeof(r.cuts));
        it = best_split.emplace(key, r).first;
      }
      const SplitResult &r = it->second;
      if (r.rc == CHM_ERR_NO_FEASIBLE) { fits = false; break; }
      cand.length[p] = len[p];
      cand.micro_batches[p] = mb[p];
      memcpy(cand.cuts[p], r.cuts, sizeof(r.cuts));
      cand.pipeline_us[p] = r.cost;
      cand.t_step_us = std::max(cand.t_step_us, r.cost);
    }
    if (!fits) continue;
    // positions of the new layout, pipeline by pipeline, stage by stage
    std::vector<int32_t> pos;
    for (int p = 0; p < dp; ++p)
      for (int j = 0; j < len[p]; ++j) {
        pos.push_back(j == 0 ? 0 : cand.cuts[p][j - 1]);
        pos.push_back(j == len[p] - 1 ? L : cand.cuts[p][j]);
      }
    if (hipMemcpyAsync(sc.d_pos, pos.data(), pos.size() * sizeof(int32_t), hipMemcpyHostToDevice, st) != hipSuccess) return CHM_ERR_HIP;
    AssignArgs a;
    a.n = N; a.L = L; a.held = sc.d_held; a.pos = sc.d_pos; a.pw = sc.d_pw; a.total = sc.d_total; a.position_of_node = sc.d_assign;
    a.rounds = (int32_t *)(sc.d_total + 1);
    if (hipEventRecord(ev.a, st) != hipSuccess) return CHM_ERR_HIP;
    hipLaunchKernelGGL(k_min_assignment, dim3(1), dim3(64), 0, st, a);
    if (hipGetLastError() != hipSuccess || hipEventRecord(ev.b, st) != hipSuccess) return CHM_ERR_HIP;
    if (hipMemcpyAsync(sc.h_total, sc.d_total, 2 * sizeof(int64_t), hipMemcpyDeviceToHost, st) != hipSuccess) return CHM_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return CHM_ERR_HIP;     // also keeps `pos` alive until the copy is done
    float ms = 0;
    if (hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess) return CHM_ERR_HIP;
    assign_ms += ms;
    cand.fetch_mib = sc.h_total[0];
    if (d->allreduce_us > 0) {
      int32_t rounds;
      memcpy(&rounds, &sc.h_total[1], sizeof(rounds));
      cand.comm_rounds = rounds;
      cand.t_step_us += (int64_t)d->allreduce_us * rounds;
    }
    cand.t_trans_us = (int64_t)d->restart_us + (int64_t)d->xfer_us_per_mib * cand.fetch_mib;
    // (H - t_trans) / t_step, larger is better; exact comparison by cross-multiplication
    const __int128 gain = (__int128)d->horizon_us - cand.t_trans_us;
    if (!have || gain * best_step > best_gain * cand.t_step_us) {
      const int32_t seen = out->n_candidates;
      *out = cand;
      out->n_candidates = seen;
      out->found = 1;
      have = true; best_gain = gain; best_step = cand.t_step_us;
    }
  }
  out->splits_scored = splits_scored;
  out->splits_feasible = splits_feasible;
  out->splits_evaluated = splits_evaluated;
  out->algorithmic_ops = algorithmic_ops;
  out->search_ms = search_ms;
  out->assign_ms = assign_ms;
  return CHM_OK;
}
}  // namespace
