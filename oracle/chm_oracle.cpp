// CPU oracle for post-failure execution-plan scoring.  TEST INFRASTRUCTURE ONLY:
// see chm_oracle.h for what it is, which passages of the paper each part follows
// and which conventions are unpinned.  Plain loops, int64 everywhere, one thread.
#include "chm_oracle.h"

#include <algorithm>
#include <cstring>
#include <vector>

namespace {

typedef unsigned __int128 u128;
typedef __int128 i128;

// ---------------------------------------------------------------------------------------
// binomials (Pascal's triangle, saturating)
// ---------------------------------------------------------------------------------------
struct Pascal {
  uint64_t c[ORC_MAX_L + 1][ORC_MAX_L + 1];
  Pascal() {
    for (int n = 0; n <= ORC_MAX_L; ++n)
      for (int k = 0; k <= ORC_MAX_L; ++k) {
        if (k > n) c[n][k] = 0;
        else if (k == 0 || k == n) c[n][k] = 1;
        else {
          uint64_t a = c[n - 1][k - 1], b = c[n - 1][k];
          c[n][k] = (a == UINT64_MAX || b == UINT64_MAX || a > UINT64_MAX - b) ? UINT64_MAX : a + b;
        }
      }
  }
};
const Pascal &pascal() { static Pascal p; return p; }

uint64_t sat_mul(uint64_t a, uint64_t b) {
  u128 p = (u128)a * b;
  return p > (u128)UINT64_MAX ? UINT64_MAX : (uint64_t)p;
}

// ---------------------------------------------------------------------------------------
// reroute vectors: non-negative integer vectors of a given length and sum, each entry
// at most cap (cap <= 0: no cap), ordered lexicographically, first entry most significant
// ---------------------------------------------------------------------------------------
struct Compositions {
  int parts, total, cap;
  std::vector<std::vector<uint64_t>> n;  // n[p][t] = vectors of length p with sum t
  Compositions(int parts_, int total_, int cap_) : parts(parts_), total(total_), cap(cap_) {
    n.assign(parts + 1, std::vector<uint64_t>(total + 1, 0));
    n[0][0] = 1;
    for (int p = 1; p <= parts; ++p)
      for (int t = 0; t <= total; ++t) {
        uint64_t acc = 0;
        for (int v = 0; v <= t; ++v) {
          if (cap > 0 && v > cap) break;
          uint64_t x = n[p - 1][t - v];
          acc = (x == UINT64_MAX || acc > UINT64_MAX - x) ? UINT64_MAX : acc + x;
        }
        n[p][t] = acc;
      }
  }
  uint64_t count() const { return n[parts][total]; }
  bool unrank(uint64_t rank, uint16_t *r) const {
    if (rank >= count()) return false;
    int rem = total;
    for (int pos = 0; pos < parts; ++pos) {
      int left = parts - 1 - pos;
      bool found = false;
      for (int v = 0; v <= rem; ++v) {
        if (cap > 0 && v > cap) break;
        uint64_t cnt = n[left][rem - v];
        if (rank < cnt) { r[pos] = (uint16_t)v; rem -= v; found = true; break; }
        rank -= cnt;
      }
      if (!found) return false;
    }
    return true;
  }
  uint64_t rank(const uint16_t *r) const {
    uint64_t acc = 0;
    int rem = total;
    for (int pos = 0; pos < parts; ++pos) {
      int left = parts - 1 - pos;
      for (int v = 0; v < r[pos]; ++v) acc += n[left][rem - v];
      rem -= r[pos];
    }
    return acc;
  }
};

}  // namespace

// ---------------------------------------------------------------------------------------
// building blocks (C interface)
// ---------------------------------------------------------------------------------------
extern "C" uint64_t orc_binom(int32_t n, int32_t k) {
  if (n < 0 || k < 0 || k > n) return 0;
  if (n > ORC_MAX_L) return UINT64_MAX;
  return pascal().c[n][k];
}

// A split of L layers into k+1 non-empty contiguous stages is the set of its cut
// positions 1 <= c_1 < ... < c_k <= L-1 (stage j = layers [c_j, c_{j+1}), c_0 = 0,
// c_{k+1} = L).  Its rank is the combinatorial number system value of {c_i - 1}.
extern "C" uint64_t orc_partition_rank(int32_t k, const uint8_t *cuts) {
  uint64_t r = 0;
  for (int i = 1; i <= k; ++i) r += orc_binom((int)cuts[i - 1] - 1, i);
  return r;
}

extern "C" void orc_partition_rank_batch(int32_t k, const uint8_t *cuts, uint64_t n, uint64_t *ranks) {
  for (uint64_t i = 0; i < n; ++i) ranks[i] = orc_partition_rank(k, cuts + i * (uint64_t)k);
}

extern "C" int orc_partition_unrank(int32_t L, int32_t k, uint64_t rank, uint8_t *cuts) {
  if (L < 1 || L > ORC_MAX_L || k < 0 || k > L - 1) return ORC_ERR_ARG;
  if (rank >= orc_binom(L - 1, k)) return ORC_ERR_RANGE;
  uint64_t rem = rank;
  for (int i = k; i >= 1; --i) {
    int x = i - 1;                         // C(i-1, i) = 0 <= rem always
    while (x + 1 <= L - 2 && orc_binom(x + 1, i) <= rem) ++x;
    cuts[i - 1] = (uint8_t)(x + 1);
    rem -= orc_binom(x, i);
  }
  return rem == 0 ? ORC_OK : ORC_ERR_RANGE;
}

extern "C" uint64_t orc_reroute_count(int32_t parts, int32_t total, int32_t cap) {
  if (parts < 0 || total < 0) return 0;
  return Compositions(parts, total, cap).count();
}
extern "C" int orc_reroute_unrank(int32_t parts, int32_t total, int32_t cap, uint64_t rank, uint16_t *r) {
  if (parts < 0 || total < 0) return ORC_ERR_ARG;
  return Compositions(parts, total, cap).unrank(rank, r) ? ORC_OK : ORC_ERR_RANGE;
}
extern "C" uint64_t orc_reroute_rank(int32_t parts, int32_t total, int32_t cap, const uint16_t *r) {
  return Compositions(parts, total, cap).rank(r);
}

// node speed factor: a time multiplier in Q16, applied to a stage sum, round half up
extern "C" int64_t orc_scale_q16(int64_t x, uint32_t q) { return (x * (int64_t)q + 32768) >> 16; }

// One pipeline under the 1F1B order.  Stage s runs min(S-1-s, M) warm-up forwards,
// then alternates forward / backward, then drains the remaining backwards.  An
// operation starts when both the previous operation of its stage and the operation
// it depends on (same micro-batch: previous stage for a forward, next stage for a
// backward, the stage's own forward for the last stage's backward) have ended.
extern "C" int64_t orc_makespan_1f1b(int32_t S, const int64_t *F, const int64_t *B, int32_t M) {
  if (S < 1 || M < 1) return 0;
  struct Op { int kind, mb; };  // kind 0 = forward, 1 = backward
  std::vector<std::vector<Op>> order(S);
  for (int s = 0; s < S; ++s) {
    int w = std::min(S - 1 - s, M);
    for (int j = 0; j < w; ++j) order[s].push_back({0, j});
    for (int j = 0; j < M - w; ++j) { order[s].push_back({0, w + j}); order[s].push_back({1, j}); }
    for (int j = M - w; j < M; ++j) order[s].push_back({1, j});
  }
  std::vector<std::vector<int64_t>> endF(S, std::vector<int64_t>(M, -1)), endB(S, std::vector<int64_t>(M, -1));
  std::vector<int64_t> clock(S, 0);
  std::vector<size_t> next(S, 0);
  size_t remaining = (size_t)2 * S * M;
  while (remaining) {
    bool progress = false;
    for (int s = 0; s < S; ++s) {
      while (next[s] < order[s].size()) {
        Op op = order[s][next[s]];
        int64_t dep;
        if (op.kind == 0) dep = (s == 0) ? 0 : endF[s - 1][op.mb];
        else              dep = (s == S - 1) ? endF[s][op.mb] : endB[s + 1][op.mb];
        if (dep < 0) break;  // dependency not produced yet
        int64_t start = std::max(clock[s], dep);
        int64_t end = start + (op.kind == 0 ? F[s] : B[s]);
        (op.kind == 0 ? endF : endB)[s][op.mb] = end;
        clock[s] = end;
        ++next[s]; --remaining; progress = true;
      }
    }
    if (!progress) return -1;  // cannot happen for a 1F1B order
  }
  return *std::max_element(clock.begin(), clock.end());
}

extern "C" int64_t orc_missing_interval(const int64_t *pw, int32_t a, int32_t b, int32_t a0, int32_t b0) {
  int64_t need = pw[b] - pw[a];
  int lo = std::max(a, a0), hi = std::min(b, b0);
  int64_t have = hi > lo ? pw[hi] - pw[lo] : 0;
  return need - have;
}

// micro-batches over pipelines in proportion to their node counts; what is left over is
// handed out one by one from the first pipeline on; a pipeline left empty takes one
// micro-batch from the largest pipeline (lowest index on ties) until none is empty.
extern "C" void orc_distribute_batch(int32_t D, int32_t total, const int32_t *nodes, int32_t *out) {
  int64_t N = 0;
  for (int d = 0; d < D; ++d) N += nodes[d];
  int64_t given = 0;
  for (int d = 0; d < D; ++d) {
    out[d] = nodes[d] > 0 ? (int32_t)((int64_t)total * nodes[d] / N) : 0;
    given += out[d];
  }
  int64_t left = total - given;
  for (int d = 0; left > 0; d = (d + 1) % D)
    if (nodes[d] > 0) { ++out[d]; --left; }
  for (;;) {
    int empty = -1, big = -1;
    for (int d = 0; d < D; ++d) {
      if (nodes[d] <= 0) continue;
      if (out[d] == 0 && empty < 0) empty = d;
      if (big < 0 || out[d] > out[big]) big = d;
    }
    if (empty < 0 || big < 0 || out[big] < 2) break;
    --out[big]; ++out[empty];
  }
}

// fault-free layout: floor(L/S) layers per stage, the L mod S extra ones on the last stages
extern "C" void orc_layout_p0(int32_t L, int32_t S, int32_t *bounds) {
  int base = L / S, extra = L % S;
  bounds[0] = 0;
  for (int s = 0; s < S; ++s) bounds[s + 1] = bounds[s] + base + (s >= S - extra ? 1 : 0);
}

// Kuhn-Munkres (Hungarian) algorithm: minimum total cost of assigning n nodes (rows) to n
// positions (columns), one to one.  Rows are added one at a time; for each new row the cheapest
// augmenting path is grown Dijkstra-style over reduced costs cost - u[row] - v[col], the
// potentials u, v are raised by the step that makes the next column tight, and the matching
// is flipped along the path once a free column is reached.
extern "C" int64_t orc_min_assignment(int32_t n, const int64_t *cost, int32_t *position_of_node) {
  if (n <= 0 || !cost) return 0;
  const int64_t BIG = INT64_MAX / 4;
  std::vector<int64_t> u(n, 0), v(n + 1, 0);
  std::vector<int> row_of_col(n + 1, -1);        // column n is the virtual start column of a new row
  for (int r = 0; r < n; ++r) {
    std::vector<int64_t> slack(n + 1, BIG);      // cheapest reduced cost seen so far into each column
    std::vector<int> prev_col(n + 1, n);         // column from which that cheapest edge leaves (via its row)
    std::vector<char> in_tree(n + 1, 0);
    row_of_col[n] = r;
    int c0 = n;
    for (;;) {
      in_tree[c0] = 1;
      const int r0 = row_of_col[c0];
      int64_t step = BIG;
      int c_next = -1;
      for (int c = 0; c < n; ++c) {
        if (in_tree[c]) continue;
        const int64_t red = cost[(size_t)r0 * n + c] - u[r0] - v[c];
        if (red < slack[c]) { slack[c] = red; prev_col[c] = c0; }
        if (slack[c] < step) { step = slack[c]; c_next = c; }
      }
      for (int c = 0; c <= n; ++c) {
        if (in_tree[c]) { u[row_of_col[c]] += step; v[c] -= step; }
        else slack[c] -= step;
      }
      c0 = c_next;
      if (row_of_col[c0] < 0) break;             // reached a free column: augment
    }
    while (c0 != n) {
      const int pc = prev_col[c0];
      row_of_col[c0] = row_of_col[pc];
      c0 = pc;
    }
  }
  int64_t total = 0;
  for (int c = 0; c < n; ++c) {
    total += cost[(size_t)row_of_col[c] * n + c];
    if (position_of_node) position_of_node[row_of_col[c]] = c;
  }
  return total;
}

extern "C" int32_t orc_comm_rounds(int32_t L, int32_t n_devices, const uint8_t *holds) {
  if (L < 1) return 0;
  std::vector<std::vector<char>> adj(L, std::vector<char>(L, 0));
  for (int dev = 0; dev < n_devices; ++dev)
    for (int a = 0; a < L; ++a)
      for (int b = 0; b < L; ++b)
        if (a != b && holds[(size_t)dev * L + a] && holds[(size_t)dev * L + b]) adj[a][b] = 1;
  std::vector<int> colour(L, -1);
  int used = 0;
  for (int l = 0; l < L; ++l) {
    std::vector<char> taken(L + 1, 0);
    for (int o = 0; o < l; ++o)
      if (adj[l][o]) taken[colour[o]] = 1;
    int c = 0;
    while (taken[c]) ++c;
    colour[l] = c;
    used = std::max(used, c + 1);
  }
  return used;
}

// ---------------------------------------------------------------------------------------
// scenario
// ---------------------------------------------------------------------------------------
struct orc_scenario {
  int L, S, D, M;
  std::vector<int64_t> fwd, bwd, mem, pf, pb, pw, pa;   // prefix sums have L+1 entries (pa: activations)
  std::vector<uint32_t> q;                              // [D*S]
  std::vector<char> failed;                             // [D*S]
  int64_t comm, cap, K, reconf[3], xfer;
  int reroute_cap;
  int transfer_assign;                                  // strategy 1: 1 = least-transfer node-to-stage assignment
  int64_t allreduce;                                    // time of one round of gradient communication, 0 = not modelled
  std::vector<int> p0;                                  // [S+1]
  // failed-node distribution
  std::vector<int> fail_in_replica, fail_in_stage;      // [D], [S]
  std::vector<int> affected;                            // stages with failures, ascending
  std::vector<std::vector<int>> peers;                  // per affected stage: surviving replicas, ascending
  std::vector<Compositions> comps;                      // per affected stage
  int SB;                                               // stages of the re-partitioned pipelines
  std::vector<int> mb_B;                                // [D] micro-batches per pipeline in family B
  bool has[3];
  orc_space space;
  uint32_t qof(int d, int s) const { return q[d * S + s]; }
  bool dead(int d, int s) const { return failed[d * S + s] != 0; }
};

namespace {

const orc_family *family_of(const orc_scenario *s, int strategy) {
  for (int i = 0; i < s->space.n_families; ++i)
    if (s->space.fam[i].strategy == strategy) return &s->space.fam[i];
  return nullptr;
}

struct StageSums { std::vector<int64_t> f, b, m, a; std::vector<int> lo; };

StageSums stage_sums(const orc_scenario *s, int k, const uint8_t *cuts) {
  StageSums r;
  r.lo.assign(k + 2, 0);
  for (int i = 1; i <= k; ++i) r.lo[i] = cuts[i - 1];
  r.lo[k + 1] = s->L;
  for (int j = 0; j <= k; ++j) {
    r.f.push_back(s->pf[r.lo[j + 1]] - s->pf[r.lo[j]]);
    r.b.push_back(s->pb[r.lo[j + 1]] - s->pb[r.lo[j]]);
    r.m.push_back(s->pw[r.lo[j + 1]] - s->pw[r.lo[j]]);
    r.a.push_back(s->pa[r.lo[j + 1]] - s->pa[r.lo[j]]);
  }
  return r;
}

// peak memory of the node at position i of an n-stage pipeline (Memory Estimator,
// eq. (peak_memory_decomposed)): static part + (n - i) micro-batches' worth of activations
int64_t peak_memory(int64_t static_mib, int64_t act_mib, int n, int i) { return static_mib + (int64_t)(n - i) * act_mib; }

bool cuts_valid(const orc_scenario *s, int k, const uint8_t *cuts) {
  int prev = 0;
  for (int i = 0; i < k; ++i) { if (cuts[i] <= prev || cuts[i] > s->L - 1) return false; prev = cuts[i]; }
  return true;
}

// step time of the fault-free layout for the replicas family B leaves untouched
// (ORC_INF when the layout itself does not fit in memory)
int64_t healthy_step_B(const orc_scenario *s) {
  int64_t t = 0;
  for (int d = 0; d < s->D; ++d) {
    if (s->fail_in_replica[d]) continue;
    std::vector<int64_t> F(s->S), B(s->S);
    for (int j = 0; j < s->S; ++j) {
      if (peak_memory(s->pw[s->p0[j + 1]] - s->pw[s->p0[j]], s->pa[s->p0[j + 1]] - s->pa[s->p0[j]], s->S, j) > s->cap) return ORC_INF;
      F[j] = orc_scale_q16(s->pf[s->p0[j + 1]] - s->pf[s->p0[j]], s->qof(d, j));
      B[j] = orc_scale_q16(s->pb[s->p0[j + 1]] - s->pb[s->p0[j]], s->qof(d, j));
    }
    t = std::max(t, orc_makespan_1f1b(s->S, F.data(), B.data(), s->mb_B[d]) + (int64_t)(s->S - 1) * s->comm);
  }
  return t;
}

// Everything of a plan's cost except the rerouting penalty.  For the rerouting family
// also returns w[a][i] = forward+backward time of affected stage a on its i-th peer.
int64_t base_cost_terms(const orc_scenario *s, int strategy, int k, const uint8_t *cuts,
                        int64_t *t_step_out, int64_t *reconf_out,
                        std::vector<std::vector<int64_t>> *w) {
  const int S = s->S;
  StageSums st = stage_sums(s, k, cuts);
  int64_t t_step = 0, missing = 0;
  if (strategy == 0) {            // redundant computation: own stage + successor's on every node
    for (int d = 0; d < s->D; ++d) {        // every surviving node holds its own stage and its successor's
      int n = S - s->fail_in_replica[d], pos = 0;
      for (int j = 0; j < S; ++j) {
        if (s->dead(d, j)) continue;
        int nx = (j + 1) % S;
        if (peak_memory(st.m[j] + st.m[nx], st.a[j] + st.a[nx], n, pos) > s->cap) return ORC_INF;
        ++pos;
      }
    }
    for (int d = 0; d < s->D; ++d) {
      std::vector<int64_t> F, B;
      for (int j = 0; j < S; ++j) {
        if (s->dead(d, j)) continue;
        int nx = (j + 1) % S;
        F.push_back(orc_scale_q16(st.f[j] + st.f[nx], s->qof(d, j)));
        B.push_back(orc_scale_q16(st.b[j] + st.b[nx], s->qof(d, j)));
      }
      int n = (int)F.size();
      t_step = std::max(t_step, orc_makespan_1f1b(n, F.data(), B.data(), s->M) + (int64_t)(n - 1) * s->comm);
    }
    for (int j = 0; j < S; ++j)
      missing += orc_missing_interval(s->pw.data(), st.lo[j], st.lo[j + 1], s->p0[j], s->p0[j + 1]);
  } else if (strategy == 1) {     // failed pipelines re-partitioned onto their surviving nodes
    const int SB = s->SB;
    for (int j = 0; j < SB; ++j) if (peak_memory(st.m[j], st.a[j], SB, j) > s->cap) return ORC_INF;
    t_step = healthy_step_B(s);
    if (t_step == ORC_INF) return ORC_INF;
    for (int d = 0; d < s->D; ++d) {
      if (!s->fail_in_replica[d]) continue;
      std::vector<int> host;      // old stage index of the node that runs new stage j
      for (int j = 0; j < S; ++j) if (!s->dead(d, j)) host.push_back(j);
      std::vector<int64_t> F(SB), B(SB);
      for (int j = 0; j < SB; ++j) {
        F[j] = orc_scale_q16(st.f[j], s->qof(d, host[j]));
        B[j] = orc_scale_q16(st.b[j], s->qof(d, host[j]));
      }
      // Cost[i][j]: MiB the i-th surviving node must fetch to hold new stage j (Restorer, "Weight Transfer")
      std::vector<int64_t> fetch((size_t)SB * SB);
      for (int i = 0; i < SB; ++i)
        for (int j = 0; j < SB; ++j)
          fetch[(size_t)i * SB + j] = orc_missing_interval(s->pw.data(), st.lo[j], st.lo[j + 1], s->p0[host[i]], s->p0[host[i] + 1]);
      int64_t miss_d = 0;
      if (s->transfer_assign) miss_d = orc_min_assignment(SB, fetch.data(), nullptr);
      else for (int j = 0; j < SB; ++j) miss_d += fetch[(size_t)j * SB + j];
      t_step = std::max(t_step, orc_makespan_1f1b(SB, F.data(), B.data(), s->mb_B[d]) + (int64_t)(SB - 1) * s->comm);
      missing = std::max(missing, miss_d);   // pipelines move their weights in parallel
    }
  } else {                        // data rerouting: every pipeline keeps S stages and M micro-batches
    for (int j = 0; j < S; ++j) if (peak_memory(st.m[j], st.a[j], S, j) > s->cap) return ORC_INF;
    for (int d = 0; d < s->D; ++d) {
      std::vector<int64_t> F(S), B(S);
      for (int j = 0; j < S; ++j) {
        uint32_t qq = s->dead(d, j) ? 65536u : s->qof(d, j);
        F[j] = orc_scale_q16(st.f[j], qq);
        B[j] = orc_scale_q16(st.b[j], qq);
      }
      t_step = std::max(t_step, orc_makespan_1f1b(S, F.data(), B.data(), s->M));
    }
    t_step += (int64_t)(S - 1) * s->comm;
    for (int j = 0; j < S; ++j)
      missing += orc_missing_interval(s->pw.data(), st.lo[j], st.lo[j + 1], s->p0[j], s->p0[j + 1]);
    if (w) {
      w->clear();
      for (size_t a = 0; a < s->affected.size(); ++a) {
        int i = s->affected[a];
        std::vector<int64_t> row;
        for (int d : s->peers[a])
          row.push_back(orc_scale_q16(st.f[i], s->qof(d, i)) + orc_scale_q16(st.b[i], s->qof(d, i)));
        w->push_back(row);
      }
    }
  }
  if (s->allreduce > 0) {
    // which layers every device holds under this plan (see the header), then the colouring
    std::vector<uint8_t> holds;
    int n_dev = 0;
    auto add_device = [&](int lo, int hi, int lo2, int hi2) {
      holds.resize((size_t)(n_dev + 1) * s->L, 0);
      for (int l = lo; l < hi; ++l) holds[(size_t)n_dev * s->L + l] = 1;
      for (int l = lo2; l < hi2; ++l) holds[(size_t)n_dev * s->L + l] = 1;
      ++n_dev;
    };
    for (int d = 0; d < s->D; ++d) {
      if (strategy == 1 && s->fail_in_replica[d]) {
        for (int j = 0; j < s->SB; ++j) add_device(st.lo[j], st.lo[j + 1], 0, 0);
        continue;
      }
      for (int j = 0; j < S; ++j) {
        if (s->dead(d, j)) continue;
        if (strategy == 0) add_device(st.lo[j], st.lo[j + 1], st.lo[(j + 1) % S], st.lo[(j + 1) % S + 1]);
        else if (strategy == 1) add_device(s->p0[j], s->p0[j + 1], 0, 0);
        else add_device(st.lo[j], st.lo[j + 1], 0, 0);
      }
    }
    t_step += s->allreduce * orc_comm_rounds(s->L, n_dev, holds.data());
  }
  *t_step_out = t_step;
  *reconf_out = s->reconf[strategy] + s->xfer * missing;
  return 0;
}

// rerouting penalty of one affected stage: the peer that finishes its extra
// micro-batches last decides the delay (extra micro-batches x that peer's stage time)
int64_t stage_penalty(const std::vector<int64_t> &w, const uint16_t *r) {
  int64_t p = 0;
  for (size_t i = 0; i < w.size(); ++i) p = std::max(p, (int64_t)r[i] * w[i]);
  return p;
}

int64_t full_cost(const orc_scenario *s, int strategy, int k, const uint8_t *cuts,
                  const std::vector<std::vector<uint16_t>> &rr /* per affected stage, per peer */,
                  int64_t *t_step_out = nullptr, int64_t *t_trans_out = nullptr) {
  int64_t t_step, reconf;
  std::vector<std::vector<int64_t>> w;
  if (t_step_out) *t_step_out = 0;
  if (t_trans_out) *t_trans_out = 0;
  if (base_cost_terms(s, strategy, k, cuts, &t_step, &reconf, &w) == ORC_INF) return ORC_INF;
  if (strategy == 2)
    for (size_t a = 0; a < s->affected.size(); ++a) t_step += stage_penalty(w[a], rr[a].data());
  if (t_step_out) *t_step_out = t_step;
  if (t_trans_out) *t_trans_out = reconf;
  return s->K * t_step + reconf;
}

void split_reroute_rank(const orc_scenario *s, uint64_t rank, std::vector<uint64_t> *per_stage) {
  size_t n = s->affected.size();
  per_stage->assign(n, 0);
  for (size_t a = n; a-- > 0;) {
    uint64_t R = s->comps[a].count();
    (*per_stage)[a] = rank % R;
    rank /= R;
  }
}

void fill_plan(const orc_scenario *s, const orc_family *f, uint64_t part_rank,
               const std::vector<uint64_t> &rr_rank, int64_t cost, orc_plan *out) {
  std::memset(out, 0, sizeof(*out));
  uint64_t joint = 0;
  for (size_t a = 0; a < rr_rank.size(); ++a) joint = joint * s->comps[a].count() + rr_rank[a];
  out->index = f->offset + part_rank * f->n_reroute + joint;
  out->cost = cost;
  out->strategy = f->strategy;
  out->stages = f->stages;
  orc_partition_unrank(s->L, f->stages - 1, part_rank, out->cuts);
  if (f->strategy == 2) {
    out->n_affected = (int)s->affected.size();
    for (size_t a = 0; a < s->affected.size(); ++a) {
      out->affected_stage[a] = s->affected[a];
      uint16_t r[ORC_MAX_DP] = {0};
      s->comps[a].unrank(rr_rank[a], r);
      for (size_t i = 0; i < s->peers[a].size(); ++i) out->reroute[a][s->peers[a][i]] = r[i];
    }
  }
}

// all valid reroute vectors of one affected stage in rank order; keeps the first minimum
struct StageSweep {
  const Compositions &c; const std::vector<int64_t> &w;
  uint16_t r[ORC_MAX_DP]; uint64_t rank = 0, best_rank = 0; int64_t best = ORC_INF;
  StageSweep(const Compositions &c_, const std::vector<int64_t> &w_) : c(c_), w(w_) {}
  void go(int pos, int rem) {
    if (pos == c.parts) {
      int64_t p = stage_penalty(w, r);
      if (p < best) { best = p; best_rank = rank; }
      ++rank;
      return;
    }
    for (int v = 0; v <= rem; ++v) {
      if (c.cap > 0 && v > c.cap) break;
      if (c.n[c.parts - 1 - pos][rem - v] == 0) continue;   // the rest cannot absorb what is left
      r[pos] = (uint16_t)v;
      go(pos + 1, rem - v);
    }
  }
};

void best_init(orc_plan *b) { std::memset(b, 0, sizeof(*b)); b->index = UINT64_MAX; b->cost = ORC_INF; }

int search_family_range(const orc_scenario *s, const orc_family *f, uint64_t first, uint64_t count,
                        orc_plan *best, uint64_t *evals, uint64_t *fitting = nullptr) {
  const int k = f->stages - 1;
  uint8_t cuts[ORC_MAX_PP];
  for (uint64_t pr = first; pr < first + count; ++pr) {
    orc_partition_unrank(s->L, k, pr, cuts);
    int64_t t_step, reconf;
    std::vector<std::vector<int64_t>> w;
    bool ok = base_cost_terms(s, f->strategy, k, cuts, &t_step, &reconf, &w) != ORC_INF;
    std::vector<uint64_t> rr_rank;
    if (f->strategy == 2) {
      uint64_t n_eval = 0;
      for (size_t a = 0; a < s->affected.size(); ++a) n_eval += s->comps[a].count();
      if (evals) *evals += s->affected.empty() ? 1 : n_eval;
      if (!ok) continue;
      if (fitting) *fitting += 1;
      for (size_t a = 0; a < s->affected.size(); ++a) {
        StageSweep sw(s->comps[a], w[a]);
        sw.go(0, s->comps[a].total);
        t_step += sw.best;
        rr_rank.push_back(sw.best_rank);
      }
    } else {
      if (evals) *evals += 1;
      if (!ok) continue;
      if (fitting) *fitting += 1;
    }
    int64_t cost = s->K * t_step + reconf;
    if (cost < best->cost) {
      fill_plan(s, f, pr, rr_rank, cost, best);
      best->t_step_us = t_step;
      best->t_trans_us = reconf;
    }
  }
  return ORC_OK;
}

}  // namespace

extern "C" int orc_open(const orc_desc *d, orc_scenario **out) {
  if (!d || !out) return ORC_ERR_ARG;
  *out = nullptr;
  if (d->L < 1 || d->L > ORC_MAX_L || d->PP < 1 || d->PP > ORC_MAX_PP || d->PP > d->L ||
      d->DP < 1 || d->DP > ORC_MAX_DP || d->M < 1 || d->M > ORC_MAX_M ||
      d->n_failed < 0 || d->n_failed > ORC_MAX_FAILED || !d->fwd_us || !d->bwd_us || !d->mem_mib ||
      (d->n_failed > 0 && !d->failed_nodes) || d->comm_us < 0 || d->mem_cap_mib < 1 ||
      d->horizon_steps < 1 || d->xfer_us_per_mib < 0 || d->transfer_assign < 0 || d->transfer_assign > 1 ||
      d->allreduce_us < 0)
    return ORC_ERR_ARG;
  for (int i = 0; i < 3; ++i) if (d->reconf_us[i] < 0) return ORC_ERR_ARG;
  orc_scenario *s = new orc_scenario();
  s->L = d->L; s->S = d->PP; s->D = d->DP; s->M = d->M;
  s->comm = d->comm_us; s->cap = d->mem_cap_mib; s->K = d->horizon_steps; s->xfer = d->xfer_us_per_mib;
  s->reroute_cap = d->reroute_cap;
  s->transfer_assign = d->transfer_assign;
  s->allreduce = d->allreduce_us;
  for (int i = 0; i < 3; ++i) s->reconf[i] = d->reconf_us[i];
  s->pf.assign(s->L + 1, 0); s->pb.assign(s->L + 1, 0); s->pw.assign(s->L + 1, 0); s->pa.assign(s->L + 1, 0);
  for (int l = 0; l < s->L; ++l) {
    if (d->fwd_us[l] < 1 || d->bwd_us[l] < 1 || d->mem_mib[l] < 0) { delete s; return ORC_ERR_ARG; }
    s->fwd.push_back(d->fwd_us[l]); s->bwd.push_back(d->bwd_us[l]); s->mem.push_back(d->mem_mib[l]);
    s->pf[l + 1] = s->pf[l] + d->fwd_us[l];
    s->pb[l + 1] = s->pb[l] + d->bwd_us[l];
    s->pw[l + 1] = s->pw[l] + d->mem_mib[l];
    if (d->act_mib && d->act_mib[l] < 0) { delete s; return ORC_ERR_ARG; }
    s->pa[l + 1] = s->pa[l] + (d->act_mib ? d->act_mib[l] : 0);
  }
  const int nodes = s->D * s->S;
  uint32_t qmax = 65536;
  for (int n = 0; n < nodes; ++n) {
    uint32_t q = d->speed_q16 ? d->speed_q16[n] : 65536u;
    if (q < 1 || q > (1u << 20)) { delete s; return ORC_ERR_ARG; }
    s->q.push_back(q); qmax = std::max(qmax, q);
  }
  s->failed.assign(nodes, 0);
  s->fail_in_replica.assign(s->D, 0); s->fail_in_stage.assign(s->S, 0);
  for (int i = 0; i < d->n_failed; ++i) {
    int n = d->failed_nodes[i];
    if (n < 0 || n >= nodes || s->failed[n]) { delete s; return ORC_ERR_ARG; }
    s->failed[n] = 1; ++s->fail_in_replica[n / s->S]; ++s->fail_in_stage[n % s->S];
  }
  s->p0.assign(s->S + 1, 0);
  orc_layout_p0(s->L, s->S, s->p0.data());

  // --- which strategies exist for this failure set ---
  // redundant computation: the ring predecessor of every failed node must be alive
  s->has[0] = s->S >= 2;
  for (int dd = 0; dd < s->D; ++dd)
    for (int j = 0; j < s->S; ++j)
      if (s->dead(dd, j) && s->dead(dd, (j + s->S - 1) % s->S)) s->has[0] = false;
  // re-partitioning: all failed pipelines keep the same, non-zero number of nodes
  s->SB = 0; s->has[1] = d->n_failed > 0;
  for (int dd = 0; dd < s->D; ++dd) {
    if (!s->fail_in_replica[dd]) continue;
    int left = s->S - s->fail_in_replica[dd];
    if (left < 1 || (s->SB && left != s->SB)) s->has[1] = false;
    s->SB = left;
  }
  if (s->has[1]) {
    std::vector<int> n_d(s->D);
    for (int dd = 0; dd < s->D; ++dd) n_d[dd] = s->S - s->fail_in_replica[dd];
    s->mb_B.assign(s->D, 0);
    orc_distribute_batch(s->D, s->D * s->M, n_d.data(), s->mb_B.data());
  }
  // rerouting: every stage keeps at least one peer, and the capped split must be possible
  s->has[2] = true;
  uint64_t n_rr = 1;
  for (int j = 0; j < s->S; ++j) {
    int Fi = s->fail_in_stage[j];
    if (Fi == 0) continue;
    if (Fi >= s->D) { s->has[2] = false; break; }
    s->affected.push_back(j);
    std::vector<int> pe;
    for (int dd = 0; dd < s->D; ++dd) if (!s->dead(dd, j)) pe.push_back(dd);
    s->peers.push_back(pe);
    s->comps.emplace_back((int)pe.size(), Fi * s->M, s->reroute_cap);
    uint64_t R = s->comps.back().count();
    if (R == 0) { s->has[2] = false; break; }
    n_rr = sat_mul(n_rr, R);
  }
  if (!s->has[2]) { s->affected.clear(); s->peers.clear(); s->comps.clear(); n_rr = 1; }

  // --- plan space ---
  std::memset(&s->space, 0, sizeof(s->space));
  uint64_t off = 0;
  bool overflow = false;
  for (int strat = 0; strat < 3; ++strat) {
    if (!s->has[strat]) continue;
    int stages = strat == 1 ? s->SB : s->S;
    uint64_t np = orc_binom(s->L - 1, stages - 1);
    uint64_t nr = strat == 2 ? n_rr : 1;
    uint64_t tot = sat_mul(np, nr);
    if (np == UINT64_MAX || nr == UINT64_MAX || tot >= (1ull << 62) || off + tot >= (1ull << 62)) { overflow = true; break; }
    orc_family &f = s->space.fam[s->space.n_families++];
    f.offset = off; f.n_part = np; f.n_reroute = nr; f.stages = stages; f.strategy = strat;
    off += tot;
  }
  s->space.n_plans = off;
  // --- cost bound: a makespan never exceeds (M+S-1) x the largest stage time ---
  i128 tot_fb = (i128)(s->pf[s->L] + s->pb[s->L]) * 2 * ((qmax + 65535) / 65536);
  i128 t_max = (i128)(s->D * s->M + s->S - 1) * tot_fb + (i128)s->S * s->comm + (i128)s->L * s->allreduce;
  i128 pen_max = (i128)ORC_MAX_FAILED * (ORC_MAX_FAILED * s->M) * tot_fb;
  i128 reconf_max = (i128)std::max(std::max(s->reconf[0], s->reconf[1]), s->reconf[2]) + (i128)s->xfer * s->pw[s->L];
  if ((i128)s->K * (t_max + pen_max) + reconf_max >= ((i128)1 << 62)) overflow = true;
  if (overflow) { delete s; return ORC_ERR_OVERFLOW; }
  *out = s;
  return ORC_OK;
}

extern "C" void orc_close(orc_scenario *s) { delete s; }

extern "C" int orc_plan_space(const orc_scenario *s, orc_space *out) {
  if (!s || !out) return ORC_ERR_ARG;
  *out = s->space;
  return ORC_OK;
}

extern "C" int orc_decode(const orc_scenario *s, uint64_t index, orc_plan *out) {
  if (!s || !out) return ORC_ERR_ARG;
  if (index >= s->space.n_plans) return ORC_ERR_RANGE;
  for (int i = 0; i < s->space.n_families; ++i) {
    const orc_family *f = &s->space.fam[i];
    uint64_t size = f->n_part * f->n_reroute;
    if (index < f->offset || index >= f->offset + size) continue;
    uint64_t local = index - f->offset;
    std::vector<uint64_t> rr;
    if (f->strategy == 2) split_reroute_rank(s, local % f->n_reroute, &rr);
    fill_plan(s, f, local / f->n_reroute, rr, 0, out);
    std::vector<std::vector<uint16_t>> vec;
    for (size_t a = 0; a < rr.size(); ++a) {
      std::vector<uint16_t> r(ORC_MAX_DP, 0);
      s->comps[a].unrank(rr[a], r.data());
      vec.push_back(r);
    }
    out->cost = full_cost(s, f->strategy, f->stages - 1, out->cuts, vec, &out->t_step_us, &out->t_trans_us);
    return ORC_OK;
  }
  return ORC_ERR_RANGE;
}

extern "C" int orc_plan_cost(const orc_scenario *s, int32_t strategy, int32_t k, const uint8_t *cuts,
                             const uint16_t *reroute, int64_t *cost) {
  if (!s || !cost || strategy < 0 || strategy > 2 || (k > 0 && !cuts)) return ORC_ERR_ARG;
  const orc_family *f = family_of(s, strategy);
  if (!f) return ORC_ERR_UNRECOVERABLE;
  if (k != f->stages - 1 || !cuts_valid(s, k, cuts)) return ORC_ERR_ARG;
  std::vector<std::vector<uint16_t>> vec;
  if (strategy == 2) {
    for (size_t a = 0; a < s->affected.size(); ++a) {
      if (!reroute) return ORC_ERR_ARG;
      std::vector<uint16_t> r;
      int sum = 0;
      for (int d : s->peers[a]) {
        uint16_t v = reroute[a * 16 + d];
        if (s->reroute_cap > 0 && v > s->reroute_cap) return ORC_ERR_ARG;
        r.push_back(v); sum += v;
      }
      if (sum != s->comps[a].total) return ORC_ERR_ARG;
      vec.push_back(r);
    }
  }
  *cost = full_cost(s, strategy, k, cuts, vec);
  return ORC_OK;
}

extern "C" int orc_score(const orc_scenario *s, uint64_t first, uint64_t count, int64_t *costs) {
  if (!s || (count && !costs)) return ORC_ERR_ARG;
  if (first > s->space.n_plans || count > s->space.n_plans - first) return ORC_ERR_RANGE;
  orc_plan p;
  for (uint64_t i = 0; i < count; ++i) {
    int rc = orc_decode(s, first + i, &p);
    if (rc != ORC_OK) return rc;
    costs[i] = p.cost;
  }
  return ORC_OK;
}

extern "C" int orc_score_ranks(const orc_scenario *s, int32_t strategy, const uint64_t *part_ranks,
                               uint64_t n, int64_t *costs) {
  if (!s || (n && (!part_ranks || !costs)) || strategy < 0 || strategy > 2) return ORC_ERR_ARG;
  const orc_family *f = family_of(s, strategy);
  if (!f) return ORC_ERR_UNRECOVERABLE;
  if (f->n_reroute != 1) return ORC_ERR_ARG;   // explicit-partition scoring has no reroute argument
  uint8_t cuts[ORC_MAX_PP];
  std::vector<std::vector<uint16_t>> vec;
  for (size_t a = 0; a < s->affected.size(); ++a) {
    std::vector<uint16_t> r(ORC_MAX_DP, 0);
    s->comps[a].unrank(0, r.data());
    vec.push_back(r);
  }
  for (uint64_t i = 0; i < n; ++i) {
    if (part_ranks[i] >= f->n_part) return ORC_ERR_RANGE;
    orc_partition_unrank(s->L, f->stages - 1, part_ranks[i], cuts);
    costs[i] = full_cost(s, strategy, f->stages - 1, cuts, vec);
  }
  return ORC_OK;
}

extern "C" int orc_search(const orc_scenario *s, uint32_t strategy_mask, orc_plan *best) {
  if (!s || !best) return ORC_ERR_ARG;
  best_init(best);
  bool any = false;
  for (int i = 0; i < s->space.n_families; ++i) {
    const orc_family *f = &s->space.fam[i];
    if (!(strategy_mask & (1u << f->strategy))) continue;
    any = true;
    search_family_range(s, f, 0, f->n_part, best, nullptr);
  }
  if (!any) return ORC_ERR_UNRECOVERABLE;
  return best->cost == ORC_INF ? ORC_ERR_NO_FEASIBLE : ORC_OK;
}

extern "C" int orc_search_range(const orc_scenario *s, int32_t strategy, uint64_t part_first,
                                uint64_t part_count, orc_plan *best, uint64_t *evals) {
  if (!s || !best) return ORC_ERR_ARG;
  const orc_family *f = family_of(s, strategy);
  if (!f) return ORC_ERR_UNRECOVERABLE;
  if (part_first > f->n_part || part_count > f->n_part - part_first) return ORC_ERR_RANGE;
  best_init(best);
  if (evals) *evals = 0;
  search_family_range(s, f, part_first, part_count, best, evals);
  return best->cost == ORC_INF ? ORC_ERR_NO_FEASIBLE : ORC_OK;
}

extern "C" int orc_search_range_counted(const orc_scenario *s, int32_t strategy, uint64_t part_first,
                                        uint64_t part_count, orc_plan *best, uint64_t *fitting) {
  if (!s || !best || !fitting) return ORC_ERR_ARG;
  const orc_family *f = family_of(s, strategy);
  if (!f) return ORC_ERR_UNRECOVERABLE;
  if (part_first > f->n_part || part_count > f->n_part - part_first) return ORC_ERR_RANGE;
  best_init(best);
  *fitting = 0;
  search_family_range(s, f, part_first, part_count, best, nullptr, fitting);
  return best->cost == ORC_INF ? ORC_ERR_NO_FEASIBLE : ORC_OK;
}

extern "C" int orc_search_joint(const orc_scenario *s, uint64_t first, uint64_t count, orc_plan *best) {
  if (!s || !best) return ORC_ERR_ARG;
  if (first > s->space.n_plans || count > s->space.n_plans - first) return ORC_ERR_RANGE;
  best_init(best);
  orc_plan p;
  for (uint64_t i = first; i < first + count; ++i) {
    orc_decode(s, i, &p);
    if (p.cost < best->cost) *best = p;
  }
  return best->cost == ORC_INF ? ORC_ERR_NO_FEASIBLE : ORC_OK;
}

// ---------------------------------------------------------------------------------------
// re-planning over DP/PP degrees (Algorithm 1)
// ---------------------------------------------------------------------------------------
extern "C" int orc_integer_partition(int32_t n, int32_t dp, int32_t pp_min, int32_t pp_max, int32_t *lengths) {
  if (dp < 1 || n < dp) return 0;
  const int base = n / dp, extra = n % dp;
  for (int p = 0; p < dp; ++p) {
    lengths[p] = base + (p >= dp - extra ? 1 : 0);
    if (lengths[p] < pp_min || lengths[p] > pp_max) return 0;
  }
  return 1;
}

extern "C" int64_t orc_best_split(int32_t L, const int32_t *fwd_us, const int32_t *bwd_us, const int32_t *mem_mib,
                                  const int32_t *act_mib, int32_t n, int32_t M, int32_t mem_cap_mib, uint8_t *cuts) {
  if (n < 1 || n > L || n > ORC_MAX_PP) return ORC_INF;
  const uint64_t count = orc_binom(L - 1, n - 1);
  int64_t best = ORC_INF;
  uint8_t c[ORC_MAX_PP];
  for (uint64_t rank = 0; rank < count; ++rank) {
    orc_partition_unrank(L, n - 1, rank, c);
    std::vector<int64_t> F(n, 0), B(n, 0);
    bool fits = true;
    for (int j = 0; j < n; ++j) {
      const int lo = j == 0 ? 0 : c[j - 1], hi = j == n - 1 ? L : c[j];
      int64_t stat = 0, act = 0;
      for (int l = lo; l < hi; ++l) {
        F[j] += fwd_us[l]; B[j] += bwd_us[l];
        stat += mem_mib[l]; act += act_mib ? act_mib[l] : 0;
      }
      if (peak_memory(stat, act, n, j) > mem_cap_mib) fits = false;
    }
    if (!fits) continue;
    const int64_t t = orc_makespan_1f1b(n, F.data(), B.data(), M);
    if (t < best) { best = t; if (cuts) std::memcpy(cuts, c, (size_t)(n - 1)); }
  }
  return best;
}

extern "C" int orc_replan(const orc_replan_desc *d, orc_replan_plan *out) {
  if (!d || !out) return ORC_ERR_ARG;
  std::memset(out, 0, sizeof(*out));
  if (d->L < 1 || d->L > ORC_MAX_L || !d->fwd_us || !d->bwd_us || !d->mem_mib || d->old_dp < 1 || d->old_dp > ORC_MAX_DP ||
      d->old_pp < 1 || d->old_pp > ORC_MAX_PP || d->old_pp > d->L || d->n_failed < 0 || (d->n_failed > 0 && !d->failed_nodes) ||
      d->dp_min < 1 || d->dp_max < d->dp_min || d->dp_max > ORC_MAX_DP || d->pp_min < 1 || d->pp_max < d->pp_min ||
      d->pp_max > ORC_MAX_PP || d->micro_batches < 1 || d->comm_us < 0 || d->mem_cap_mib < 1 || d->horizon_us < 1 ||
      d->restart_us < 0 || d->xfer_us_per_mib < 0 || d->allreduce_us < 0)
    return ORC_ERR_ARG;
  for (int l = 0; l < d->L; ++l)
    if (d->fwd_us[l] < 1 || d->bwd_us[l] < 1 || d->mem_mib[l] < 0 || (d->act_mib && d->act_mib[l] < 0)) return ORC_ERR_ARG;
  const int old_nodes = d->old_dp * d->old_pp;
  std::vector<char> dead(old_nodes, 0);
  for (int i = 0; i < d->n_failed; ++i) {
    const int n = d->failed_nodes[i];
    if (n < 0 || n >= old_nodes || dead[n]) return ORC_ERR_ARG;
    dead[n] = 1;
  }
  std::vector<int> p0(d->old_pp + 1);
  orc_layout_p0(d->L, d->old_pp, p0.data());
  std::vector<int64_t> pw(d->L + 1, 0);
  for (int l = 0; l < d->L; ++l) pw[l + 1] = pw[l] + d->mem_mib[l];
  std::vector<int> held_lo, held_hi;            // what every surviving node holds, in node-id order
  for (int n = 0; n < old_nodes; ++n)
    if (!dead[n]) { held_lo.push_back(p0[n % d->old_pp]); held_hi.push_back(p0[n % d->old_pp + 1]); }
  const int N = (int)held_lo.size();

  bool have = false;
  i128 best_gain = 0;                           // H - t_trans of the best candidate so far
  int64_t best_step = 1;
  for (int dp = d->dp_min; dp <= d->dp_max; ++dp) {
    int32_t len[ORC_MAX_DP], mb[ORC_MAX_DP];
    if (!orc_integer_partition(N, dp, d->pp_min, d->pp_max, len)) continue;
    bool usable = d->micro_batches >= dp;
    for (int p = 0; p < dp; ++p) usable = usable && len[p] <= d->L;
    if (!usable) continue;
    orc_distribute_batch(dp, d->micro_batches, len, mb);
    // a pipeline runs at most ORC_MAX_M micro-batches (the limit of the scenario path): a layout that would give
    // one more is not a candidate
    for (int p = 0; p < dp; ++p) usable = usable && mb[p] <= ORC_MAX_M;
    if (!usable) continue;
    ++out->n_candidates;
    orc_replan_plan cand;
    std::memset(&cand, 0, sizeof(cand));
    cand.dp = dp;
    bool fits = true;
    for (int p = 0; p < dp && fits; ++p) {
      cand.length[p] = len[p]; cand.micro_batches[p] = mb[p];
      const int64_t t = orc_best_split(d->L, d->fwd_us, d->bwd_us, d->mem_mib, d->act_mib, len[p], mb[p], d->mem_cap_mib, cand.cuts[p]);
      if (t == ORC_INF) { fits = false; break; }
      cand.pipeline_us[p] = t + (int64_t)(len[p] - 1) * d->comm_us;
      cand.t_step_us = std::max(cand.t_step_us, cand.pipeline_us[p]);
    }
    if (!fits) continue;
    // positions of the new layout, pipeline by pipeline, stage by stage
    std::vector<int> pos_lo, pos_hi;
    for (int p = 0; p < dp; ++p)
      for (int j = 0; j < len[p]; ++j) {
        pos_lo.push_back(j == 0 ? 0 : cand.cuts[p][j - 1]);
        pos_hi.push_back(j == len[p] - 1 ? d->L : cand.cuts[p][j]);
      }
    if (d->allreduce_us > 0) {                // one device per position of the new layout
      std::vector<uint8_t> holds((size_t)N * d->L, 0);
      for (int j = 0; j < N; ++j)
        for (int l = pos_lo[j]; l < pos_hi[j]; ++l) holds[(size_t)j * d->L + l] = 1;
      cand.comm_rounds = orc_comm_rounds(d->L, N, holds.data());
      cand.t_step_us += (int64_t)d->allreduce_us * cand.comm_rounds;
    }
    std::vector<int64_t> fetch((size_t)N * N);
    for (int i = 0; i < N; ++i)
      for (int j = 0; j < N; ++j)
        fetch[(size_t)i * N + j] = orc_missing_interval(pw.data(), pos_lo[j], pos_hi[j], held_lo[i], held_hi[i]);
    cand.fetch_mib = orc_min_assignment(N, fetch.data(), nullptr);
    cand.t_trans_us = d->restart_us + (int64_t)d->xfer_us_per_mib * cand.fetch_mib;
    // (H - t_trans) / t_step, larger is better; exact comparison by cross-multiplication
    const i128 gain = (i128)d->horizon_us - cand.t_trans_us;
    if (!have || gain * best_step > best_gain * cand.t_step_us) {
      const int32_t seen = out->n_candidates;
      *out = cand;
      out->n_candidates = seen;
      out->found = 1;
      have = true; best_gain = gain; best_step = cand.t_step_us;
    }
  }
  return ORC_OK;
}
