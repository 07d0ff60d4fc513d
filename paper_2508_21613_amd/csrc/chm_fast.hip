// Shape-specialised exhaustive search kernels of libchm for gfx950 (wave64, plain VALU
// integer work: the path is a max-plus recurrence, not a dense contraction, so no MFMA).
//
// One lane owns a run of consecutive partition ranks.  It unranks the first one
// (combinatorial number system), then walks to each next partition with a branch-free
// successor step, so unranking is amortised over the run.  Everything a plan needs lives
// in registers: the cut positions, the per-stage sums (read from one LDS table of prefix
// sums staged once per workgroup), and the recurrence frontier - ONE value per stage, see
// the evaluation order described in chm_kernels.hip.  The recurrence is unrolled over the
// (compile-time) pipeline length and runs in the frame of the forward chain (makespan32): a
// round of N forwards and N backwards is N-1 v_max_i32 and N v_add_u32.
// All values are int32: the host only selects these kernels when its load-time bound shows
// that no intermediate can reach 2^31, in which case the results equal the int64 ones.
//
// Data rerouting: after the base step time of a partition, every valid reroute vector of
// every stage that lost nodes is scored (extra micro-batches x peer stage time, max over
// peers); the vectors are read from a rank-ordered table through uniform (scalar) loads.
//
// Argmin: per lane a running (cost, run position) with strict less-than, so the lowest
// index wins inside a lane; then a DPP/shuffle wave reduction of the packed 64-bit key
// (cost << idx_bits | chunk-local partition index), one LDS step per workgroup and one
// 64-bit atomicMin per workgroup.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <type_traits>
#include <vector>

#include "chm_fast.h"
#include "chm_pool.h"

// typed front ends of the caching allocator (chm_pool.h)
template <typename T>
static inline bool pool_take(T *&p, size_t bytes) { p = (T *)pool_device_alloc(bytes); return p != nullptr; }
template <typename T>
static inline bool pool_take_pinned(T *&p, size_t bytes) { p = (T *)pool_pinned_alloc(bytes); return p != nullptr; }

namespace {

constexpr int BLOCK = 256;

// The scenario tables are never written while a search kernel runs.  Reading them through the
// constant address space tells the compiler so: uniform reads become scalar loads (wide
// s_load_dwordx16 for the reroute rows) even though the kernel also stores costs to global memory.
#define CHM_CONST __attribute__((address_space(4)))
typedef const CHM_CONST DevScenario *ScnPtr;
typedef const CHM_CONST FastTables *TabPtr;
typedef const CHM_CONST FastFamily *FamPtr;
typedef const CHM_CONST FastClass *ClsPtr;
typedef const CHM_CONST uint32_t *RowPtr;
template <typename T>
__device__ __forceinline__ const CHM_CONST T *as_const(const T *p) {
  return (const CHM_CONST T *)(uintptr_t)p;
}

__device__ __forceinline__ int imax32(int a, int b) { return a > b ? a : b; }
__device__ __forceinline__ int imin32(int a, int b) { return a < b ? a : b; }

// (x*q + 32768) >> 16 for 0 <= x < 2^31, q <= 2^20, result < 2^31
__device__ __forceinline__ int scale32(int x, uint32_t q) {
  return (int)(((uint64_t)(uint32_t)x * q + 32768u) >> 16);
}

// lower bound of scale32(f, q') + scale32(b, q') for any q' >= q, given x = f + b: each rounding loses less
// than one, so the sum is at least floor(x * q / 65536) - 1
__device__ __forceinline__ int scale_floor(int x, uint32_t q) {
  return q == 65536u ? x : imax32(0, (int)(((uint64_t)(uint32_t)x * q) >> 16) - 1);
}

// forward + backward time of a stage on a peer with factor q (uniform): nominal peers need no scaling
__device__ __forceinline__ uint32_t peer_time(int f, int b, uint32_t q) {
  return q == 65536u ? (uint32_t)(f + b) : (uint32_t)(scale32(f, q) + scale32(b, q));
}

// 1F1B pipeline time of N stages, M micro-batches; F, B per stage.  Round t: forward t on all
// stages in stage order, then backward t-(N-1-s) on stage s (see chm_kernels.hip).  The clocks are
// kept relative to the forward chain: e[s] = (time stage s is free) - (F[0] + ... + F[s-1]).  In
// that frame the forward of stage s ends at x[s] = max(e[s], x[s-1]) with no add at all, and the
// backward that stage s-1 runs right after its own forward takes the max of the same two values,
// so it leaves e[s-1] = x[s] + (F[s-1] + B[s-1]).  A round of N forwards and N backwards is N-1
// v_max_i32 and N v_add_u32.  The cool-down rounds (backwards only) run on plain clocks again.
template <int N>
__device__ __forceinline__ int makespan32(const int (&F)[N], const int (&B)[N], int M) {
  if (N == 1) return M * (F[0] + B[0]);
  if (M >= N - 1) {
    // e[s] = (time stage s is free) - (forward time of stages 0..s-1); C = forward + backward of a stage
    int e[N], C[N];
#pragma unroll
    for (int s = 0; s < N; ++s) C[s] = F[s] + B[s];
    // round 0: forward 0 runs down the empty pipeline, the last stage follows it with backward 0
#pragma unroll
    for (int s = 0; s < N; ++s) e[s] = s == N - 1 ? C[s] : F[s];
    // warm-up rounds 1..N-2: every stage runs a forward, stages >= N-1-t also a backward
#pragma unroll
    for (int t = 1; t < N - 1; ++t) {
      int x = e[0];
#pragma unroll
      for (int s = 1; s < N; ++s) {
        const int xs = imax32(e[s], x);
        e[s - 1] = (s - 1 >= N - 1 - t) ? xs + C[s - 1] : x + F[s - 1];
        x = xs;
      }
      e[N - 1] = x + C[N - 1];
    }
    // steady rounds: one forward and one backward on every stage
    for (int t = (N - 1 > 1 ? N - 1 : 1); t < M; ++t) {
      int x = e[0];
#pragma unroll
      for (int s = 1; s < N; ++s) {
        x = imax32(e[s], x);
        e[s - 1] = x + C[s - 1];
      }
      e[N - 1] = x + C[N - 1];
    }
    // back to plain clocks, then the cool-down rounds: backwards only, stage s while s <= N-2-u
    int E[N];
    int pf = 0;
#pragma unroll
    for (int s = 0; s < N; ++s) { E[s] = e[s] + pf; pf += F[s]; }
#pragma unroll
    for (int u = 0; u < N - 1; ++u) {
#pragma unroll
      for (int s = 0; s < N - 1 - u; ++s) E[s] = imax32(E[s], E[s + 1]) + B[s];
    }
    return E[0];
  }
  int E[N];
#pragma unroll
  for (int s = 0; s < N; ++s) E[s] = 0;
  // fewer micro-batches than warm-up slots: plain clocks, rounds with (uniform) predicates
  for (int t = 0; t < M + N - 1; ++t) {
    const bool fwd = t < M;
    int x = 0;
#pragma unroll
    for (int s = 0; s < N; ++s) {
      const int old = E[s];
      if (fwd) {
        E[s] = imax32(E[s], x) + F[s];
        x = E[s];
        if (s == N - 1) E[s] += B[s];
      }
      if (s >= 1) {
        const int j = t - N + s;
        if (j >= 0 && j < M) E[s - 1] = imax32(E[s - 1], old) + B[s - 1];
      }
    }
  }
  return E[0];
}

template <int N>
__device__ __forceinline__ int class_time(ClsPtr c, int (&F)[N], int (&B)[N]) {
  if (!c->unit) {
#pragma unroll
    for (int j = 0; j < N; ++j) {
      F[j] = scale32(F[j], c->q[j]);
      B[j] = scale32(B[j], c->q[j]);
    }
  }
  return makespan32<N>(F, B, c->M) + c->comm_total;
}

// The least of max_i r_i * w_i over all valid reroute vectors (r_i <= cap, sum = orphans) without looking at
// them: some vector stays within v exactly when sum_i min(cap, floor(v / w_i)) >= orphans, the sum grows with
// v, and the least such v, found by bisection, is the minimum (see k_least_penalty).  Penalties are below 2^31
// wherever these kernels run (load-time bound), so 32-bit divisions do.
__device__ __forceinline__ uint32_t least_penalty32(const uint32_t (&w)[FAST_MAX_P], int peers, uint32_t orphans, uint32_t cap) {
  uint32_t w_max = 1;
#pragma unroll
  for (int i = 0; i < FAST_MAX_P; ++i) w_max = (i < peers && w[i] > w_max) ? w[i] : w_max;
  const uint64_t all = (uint64_t)orphans * w_max;
  uint32_t lo = 0, hi = all > 0x7fffffffull ? 0x7fffffffu : (uint32_t)all;
  while (lo < hi) {
    const uint32_t v = lo + (hi - lo) / 2;
    uint32_t room = 0;
#pragma unroll
    for (int i = 0; i < FAST_MAX_P; ++i) {
      if (i < peers) {
        const uint32_t fit = w[i] == 0 ? cap : v / w[i];
        room += fit < cap ? fit : cap;
      }
    }
    if (room >= orphans) hi = v;
    else lo = v + 1;
  }
  return lo;
}

// min over all reroute vectors of one stage of max_i r_i * w_i, run by run (see FastTables):
// within a run only the last two entries change, by +1 and -1, so their products are carried
// by an add and a subtract and every vector costs those two, one v_max3_u32 and a share of a
// v_min3_u32.  Runs are read through scalar loads; all control flow is uniform.
template <int P>
__device__ __forceinline__ uint32_t sweep_runs(RowPtr runs, uint32_t n_runs, const uint32_t (&w)[P]) {
  uint32_t best = 0xffffffffu;
  if (P == 1) {                       // a single peer takes everything: one vector, one run of length 1
    if (n_runs) best = __umul24(runs[6] >> 16, w[0]);
    return best;
  }
  constexpr int Q = P >= 2 ? P - 2 : 0;
  const uint32_t wa = w[P >= 2 ? P - 2 : 0], wb = w[P - 1];
  if (n_runs == 0) return best;
  // the descriptor of the next run is fetched while the current one is swept
  uint32_t d[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) d[i] = runs[i];
  for (uint32_t r = 0; r < n_runs; ++r) {
    uint32_t nx[8];
    RowPtr nd = runs + (size_t)(r + 1 < n_runs ? r + 1 : r) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) nx[i] = nd[i];
    uint32_t pre = 0;
#pragma unroll
    for (int i = 0; i < Q; ++i) {
      const uint32_t v = __umul24(d[i], w[i]);
      pre = pre > v ? pre : v;
    }
    const uint32_t lo = d[6] & 0xffffu, rem = d[6] >> 16;
    uint32_t cnt = d[7];
    uint32_t x = __umul24(lo, wa), y = __umul24(rem - lo, wb);
    // the shared entries' maximum is the same for the whole run: it is folded in once, after the
    // minimum over the run of max(x, y).  The two products are stepped with one add and one
    // subtract per vector (kept as written: the compiler would otherwise rebuild each of them
    // from multiples of the step, which costs more instructions).
    uint32_t run_best = 0xffffffffu;
    for (; cnt >= 4; cnt -= 4) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t pen = x > y ? x : y;
        run_best = run_best < pen ? run_best : pen;
        asm volatile("v_add_u32 %0, %0, %2\n\tv_sub_u32 %1, %1, %3" : "+v"(x), "+v"(y) : "v"(wa), "v"(wb));
      }
    }
    for (; cnt > 0; --cnt) {
      const uint32_t pen = x > y ? x : y;
      run_best = run_best < pen ? run_best : pen;
      x += wa;
      y -= wb;
    }
    run_best = run_best > pre ? run_best : pre;
    best = best < run_best ? best : run_best;
#pragma unroll
    for (int i = 0; i < 8; ++i) d[i] = nx[i];
  }
  return best;
}

// min over ALL vectors of P non-negative entries summing to T (no cap) of max_i r_i * w_i, with the vector
// loop unrolled at compile time: the products r * w_i (r = 0..T) of the last two peers are built once with
// adds, the first peer's product is carried along its (outer) loop, after which a vector costs one
// v_max3_u32 (two peers: v_max_u32) and half a v_min3_u32.  For P = 2, 3 and small T.
template <int P, int T>
__device__ __forceinline__ uint32_t sweep_products(const uint32_t (&w)[P]) {
  static_assert(P == 2 || P == 3, "two or three peers");
  uint32_t last[T + 1], mid[P == 3 ? T + 1 : 1];
  last[0] = 0;
  mid[0] = 0;
#pragma unroll
  for (int r = 1; r <= T; ++r) {
    last[r] = last[r - 1] + w[P - 1];
    if (P == 3) mid[r] = mid[r - 1] + w[1];
  }
  uint32_t best = 0xffffffffu, first = 0;
#pragma unroll
  for (int r0 = 0; r0 <= T; ++r0) {
    if (P == 2) {
      const uint32_t b = last[T - r0];
      const uint32_t pen = first > b ? first : b;
      best = best < pen ? best : pen;
    } else {
#pragma unroll
      for (int r1 = 0; r1 <= T - r0; ++r1) {
        const uint32_t b = mid[P == 3 ? r1 : 0], c = last[T - r0 - r1];
        uint32_t pen = first > b ? first : b;
        pen = pen > c ? pen : c;
        best = best < pen ? best : pen;
      }
    }
    first += w[0];
  }
  return best;
}

__device__ __forceinline__ uint64_t umin64(uint64_t a, uint64_t b) { return a < b ? a : b; }

// 1-based position of the n-th set bit of x (1 <= n <= popcount(x)): which half holds it is decided
// by a population count, six times
__device__ __forceinline__ int nth_set_bit(uint64_t x, int n) {
  const uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
  int c = __popc(lo);
  bool up = n > c;
  uint32_t w = up ? hi : lo;
  int r = up ? n - c : n;
  int pos = up ? 32 : 0;
#pragma unroll
  for (int sh = 16; sh >= 1; sh >>= 1) {
    const uint32_t part = w & ((1u << sh) - 1u);
    c = __popc(part);
    up = r > c;
    w = up ? (w >> sh) : part;
    r = up ? r - c : r;
    pos += up ? sh : 0;
  }
  return pos + 1;
}

// Rounds of gradient communication under redundant computation (see comm_rounds in chm_kernels.hip):
// the colour set of stage s = the n_s lowest colours not used by stage s-1 (if its node exists) nor,
// for the last stage, by stage 0 (if the last node exists); sets are 64-bit masks, L <= 64.
template <int SP>
__device__ __forceinline__ int ring_rounds(const int (&c)[SP + 1], uint32_t node_exists) {
  uint64_t prev = 0, first = 0;
  int rounds = 0;
#pragma unroll
  for (int s = 0; s < SP; ++s) {
    const int n = c[s + 1] - c[s];
    uint64_t f = 0;
    if (s >= 1) f |= ((node_exists >> (s - 1)) & 1u) ? prev : 0ull;
    if (s >= 1 && s == SP - 1) f |= ((node_exists >> s) & 1u) ? first : 0ull;
    const int p = nth_set_bit(~f, n);
    const uint64_t low = p >= 64 ? ~0ull : ((1ull << p) - 1ull);
    const uint64_t cur = ~f & low;
    rounds = imax32(rounds, p);
    if (s == 0) first = cur;
    prev = cur;
  }
  return rounds;
}

template <int CTRL>
__device__ __forceinline__ uint64_t dpp_min(uint64_t v) {
  const int lo = __builtin_amdgcn_update_dpp((int)(uint32_t)v, (int)(uint32_t)v, CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp((int)(uint32_t)(v >> 32), (int)(uint32_t)(v >> 32), CTRL, 0xF, 0xF, false);
  return umin64(v, ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

__device__ __forceinline__ uint64_t wave_min(uint64_t v) {
  v = dpp_min<0xB1>(v);     // quad_perm [1,0,3,2]
  v = dpp_min<0x4E>(v);     // quad_perm [2,3,0,1]
  v = dpp_min<0x141>(v);    // row_half_mirror
  v = dpp_min<0x140>(v);    // row_mirror
  v = umin64(v, __shfl_xor(v, 16, 64));
  v = umin64(v, __shfl_xor(v, 32, 64));
  return v;
}

// Combinadic digits of `rem` (a partition rank): for i = K..1 the largest x with C(x, i) <= rem.
// C(., i) grows with x, so each digit is found by a four-way search over [i-1, previous digit - 1]:
// three independent table probes per step, the range shrinks to a quarter; all lanes take the same
// number of steps (no divergence), `steps` = 3 for up to 64 candidates, 4 for up to 256.
template <int K>
__device__ __forceinline__ void unrank_digits(uint64_t rem, int L, int steps, const uint64_t *table, int (&c)[K + 2]) {
  // table[(i-1) * DEV_MAX_L + x] = C(x, i)
  auto column = [table](int i, int x) { return table[(i - 1) * DEV_MAX_L + x]; };
  int hi = L - 2;
#pragma unroll
  for (int i = K; i >= 1; --i) {
    int lo = i - 1;                                  // C(i-1, i) = 0 <= rem always
    for (int s = 0; s < steps; ++s) {
      const int q = (hi - lo + 4) >> 2;              // ceil((range size) / 4), 0 only when hi < lo
      const int m1 = lo + q, m2 = m1 + q, m3 = m2 + q;
      const bool a1 = m1 <= hi && column(i, m1 <= hi ? m1 : hi) <= rem;
      const bool a2 = m2 <= hi && column(i, m2 <= hi ? m2 : hi) <= rem;
      const bool a3 = m3 <= hi && column(i, m3 <= hi ? m3 : hi) <= rem;
      // the answer lies in [lo, m1-1], [m1, m2-1], [m2, m3-1] or [m3, hi]
      const int nlo = a3 ? m3 : (a2 ? m2 : (a1 ? m1 : lo));
      const int nhi = a3 ? hi : (a2 ? m3 - 1 : (a1 ? m2 - 1 : m1 - 1));
      lo = nlo;
      hi = nhi < hi ? nhi : hi;
    }
    c[i] = lo + 1;
    rem -= column(i, lo);
    hi = lo - 1;
  }
}

// largest peak memory over the nodes of a plan: static + (pipeline length - position) * activations of the
// most demanding node of every stage (strategy 0: a node holds its stage and its ring successor's)
template <int SP, int STRAT>
__device__ __forceinline__ int largest_peak(FamPtr ff, const int (&ms)[SP], const int (&as)[SP]) {
  int mmax = 0;
  if (ff->has_act) {
#pragma unroll
    for (int j = 0; j < SP; ++j) {
      const int coef = ff->mem_coef[j];
      const int st = STRAT == 0 ? ms[j] + ms[(j + 1) % SP] : ms[j];
      const int ac = STRAT == 0 ? as[j] + as[(j + 1) % SP] : as[j];
      const int m = st + (int)__umul24((uint32_t)ac, (uint32_t)(coef < 0 ? 0 : coef));
      mmax = imax32(mmax, coef < 0 ? 0 : m);
    }
  } else {
#pragma unroll
    for (int j = 0; j < SP; ++j) {
      const int m = STRAT == 0 ? ms[j] + ms[(j + 1) % SP] : ms[j];
      mmax = imax32(mmax, ff->mem_coef[j] < 0 ? 0 : m);
    }
  }
  return mmax;
}

// Lower bound of a plan's cost from its cuts c[0..SP] and the forward + backward time cs[] of its stages.
template <int SP, int STRAT>
__device__ __forceinline__ uint64_t cost_lower_bound(ScnPtr scn, TabPtr tab, FamPtr ff, const int (&cs)[SP], const int (&c)[SP + 1]) {
    // Lower bound of the plan's cost.  Every stage of a pipeline runs its M forwards and M backwards one
    // after the other, so the pipeline takes at least M x the largest (forward + backward) of its chain;
    // rounds of gradient communication: at least the layers of the largest stage; a stage that lost
    // nodes leaves some peer with at least ceil(orphans / peers) extra micro-batches; the weight transfer
    // is at least zero.  Above the incumbent the partition can neither win nor tie.
    // (Sharper where the times allow 24-bit multiplies: stage s cannot start before the forwards of the
    // stages ahead of it and is followed by their backwards: M x its own time + the times of stages 0..s-1.)
    int lb = ff->fixed_step;
    if (STRAT == 0) {
      int cd[SP];
#pragma unroll
      for (int j = 0; j < SP; ++j) cd[j] = cs[j] + cs[(j + 1) % SP];
      for (int ci = 0; ci < ff->n_cls; ++ci) {
        const ClsPtr cl = &ff->cls[ci];
        int v = 0;
        if (ff->lb_prefix) {
          int pre = 0;
#pragma unroll
          for (int j = 0; j < SP; ++j) {
            const int cj = (j == cl->dead0 || j == cl->dead1) ? 0 : cd[j];
            v = imax32(v, (int)__umul24((uint32_t)cl->M, (uint32_t)cj) + pre);
            pre += cj;
          }
        } else {
#pragma unroll
          for (int j = 0; j < SP; ++j) v = imax32(v, (j == cl->dead0 || j == cl->dead1) ? 0 : cd[j]);
          v *= cl->M;
        }
        lb = imax32(lb, imax32(0, scale_floor(v, cl->q_min) - cl->lb_slack) + cl->comm_total);
      }
    } else {
      for (int ci = 0; ci < ff->n_cls; ++ci) {
        const ClsPtr cl = &ff->cls[ci];
        int v = 0;
        if (ff->lb_prefix) {
          int pre = 0;
#pragma unroll
          for (int j = 0; j < SP; ++j) {
            v = imax32(v, (int)__umul24((uint32_t)cl->M, (uint32_t)cs[j]) + pre);
            pre += cs[j];
          }
        } else {
#pragma unroll
          for (int j = 0; j < SP; ++j) v = imax32(v, cs[j]);
          v *= cl->M;
        }
        lb = imax32(lb, imax32(0, scale_floor(v, cl->q_min) - cl->lb_slack) + cl->comm_total);
      }
    }
    if (ff->allreduce > 0) {
      int layers = STRAT == 0 ? 0 : ff->fixed_layers;
#pragma unroll
      for (int j = 0; j < SP; ++j) layers = imax32(layers, c[j + 1] - c[j]);
      lb += ff->allreduce * layers;
    }
    if (STRAT == 2) {
      for (int st = 0; st < scn->n_aff; ++st) {
        const int sa = scn->aff_stage[st];
        int c_st = cs[0];
#pragma unroll
        for (int j = 1; j < SP; ++j) c_st = sa == j ? cs[j] : c_st;
        lb += (int)tab->lb_mult[st] * scale_floor(c_st, tab->lb_q[st]);
      }
    }
    return (uint64_t)scn->K * (uint32_t)lb + (uint64_t)scn->reconf[STRAT];
}

struct FastLaunch {
  SearchLaunch s;
  const FastTables *tab;
  const uint32_t *vecs;
  const uint32_t *runs;
  uint32_t per_lane;            // consecutive partition ranks per lane
  // split rerouting path: instead of sweeping the reroute vectors itself the kernel stores, per
  // partition, the cost without penalties and the peer stage times (null: fused sweep)
  uint64_t *base_out;
  uint32_t *weights_out;
  // compacted list mode: workgroup b owns slots [b * per_lane * BLOCK, ...) of cut_list / cut_pos, of which the
  // first cut_count[b] are filled (by k_list_filter, with the list entries that fit in memory).  In round `it`
  // lane t evaluates slot it * BLOCK + t: the partition whose cut positions are the bytes of cut_list[slot],
  // reported under list position cut_pos[slot].  Every lane of every wave has work except in a workgroup's
  // last round (null: other modes)
  const uint4 *cut_list;
  const uint32_t *cut_pos;
  const uint32_t *cut_count;
  // QUEUED kernels of the rerouting strategy: least penalty per stage from the peers' capacities instead of a sweep
  int32_t capacity_penalty = 0;
};

// Entries of a wave's queue of partitions that fit (QUEUED kernels): a ring of twice the wave width,
// since a round appends at most 64 entries to fewer than 64 waiting ones.
constexpr int QCAP = 128;

// Waves per SIMD the register allocator is asked to keep possible: up to 8 stages the kernels fit 96
// vector registers (5 waves); deeper pipelines hold more live stage sums and clocks: asked for 3 waves they take
// 98-112 registers at 9-10 stages (4 waves), 135-163 at 11-14 and 168 with a dozen spilled at 15-16 (left alone
// the allocator used 147-209, 2 waves at 16 stages).
//
// QUEUED (range search of strategies 0 and 1 without cost store): lanes whose partition fails the memory
// filter would idle through the recurrence of their wave, and consecutive ranks share their upper cuts, so
// whole runs of a lane fail together.  Each wave therefore first only filters: every lane takes the next
// partition of its run, and those that fit are appended (cut positions packed into bytes, position) to a
// ring in LDS that belongs to the wave.  Whenever 64 entries wait, the wave evaluates them, one per lane,
// with every lane busy; what is left after the last round is evaluated by a partly filled wave.  A ring is
// written and read by one wave only, whose LDS operations complete in order: no barrier is needed.
// MODE 0: every lane evaluates its own partitions; 1: QUEUED; 2: QUEUED with the bounds of a bounded search (a
// variant of its own: the bounds cost the plain queued kernel registers it does not have, 36 instead of 16
// spilled bytes per lane at 8 stages and 4 % of its time).
template <int SP, int STRAT, int MODE = 0>
__global__ void __launch_bounds__(BLOCK) __attribute__((amdgpu_waves_per_eu(SP <= 8 ? 5 : 3)))
k_fast_search(FastLaunch a) {
  constexpr bool QUEUED = MODE >= 1;
  constexpr int K = SP - 1;
  __shared__ uint4 q_cuts[QUEUED ? (BLOCK / 64) * QCAP : 1];
  __shared__ uint32_t q_pos[QUEUED ? (BLOCK / 64) * QCAP : 1];
  __shared__ int4 T[DEV_MAX_L + 1];            // prefix sums: forward, backward, static memory, activation memory
  __shared__ uint64_t BN[(K > 0 ? K : 1) * DEV_MAX_L];   // BN[(i-1)*128 + x] = C(x, i), i = 1..K
  __shared__ uint64_t wave_keys[BLOCK / 64];
  __shared__ uint32_t wave_fit[BLOCK / 64];
  __shared__ uint32_t wave_eval[BLOCK / 64];
  extern __shared__ int64_t cost_tile[];       // BLOCK * per_lane costs when a cost store with per_lane > 1 is asked for
  const ScnPtr scn = as_const(a.s.scn);
  const TabPtr tab = as_const(a.tab);
  const FamPtr ff = &tab->fam[STRAT];
  const int L = scn->L;
  const bool compact = !QUEUED && a.cut_list != nullptr;
  const uint32_t n_slots = compact ? a.cut_count[blockIdx.x] : 0u;       // filled slots of this workgroup's region
  if (compact && n_slots == 0) return;
  for (int i = threadIdx.x; i <= L; i += BLOCK) T[i] = make_int4((int)scn->pf[i], (int)scn->pb[i], (int)scn->pw[i], (int)scn->pa[i]);
  if (!compact)                                                 // a compacted list needs no unranking
    for (int i = threadIdx.x; i < K * DEV_MAX_L; i += BLOCK) BN[i] = scn->binom[1 + i / DEV_MAX_L][i % DEV_MAX_L];
  __syncthreads();

  const uint32_t lane_id = blockIdx.x * BLOCK + threadIdx.x;
  const uint32_t run_first = lane_id * a.per_lane;                       // chunk-local (a chunk holds at most 2^30 partitions)
  const uint32_t run_len = (compact || run_first >= a.s.part_count) ? 0u
                           : (uint32_t)(a.s.part_count - run_first < a.per_lane ? a.s.part_count - run_first : a.per_lane);
  const uint32_t region = blockIdx.x * a.per_lane * BLOCK;               // compact mode: first slot of this workgroup

  // cut positions c[1..K]; c[0] = 0 and c[SP] = L are constants
  int c[SP + 1];
  c[0] = 0;
  c[SP] = L;
  bool listed_ok = true;
  if (!compact) {
    uint64_t rem = run_len ? a.s.part_first + run_first + (run_first >= a.s.jump_at ? a.s.jump_by : 0) : 0;   // idle lanes walk from rank 0: always valid cuts
    if (!QUEUED && a.s.ranks != nullptr && run_len) {            // list mode (one partition per lane)
      rem = a.s.ranks[run_first];
      listed_ok = rem < scn->fam[STRAT].n_part;
      if (!listed_ok) rem = 0;
    }
    // combinadic digits from the LDS copy of the binomial table
    unrank_digits<K>(rem, L, (L - 1) <= 64 ? 3 : 4, BN, c);
  }

  const int cap = (int)scn->cap;
  uint64_t best_cost = ~0ull;
  uint32_t best_pos = 0;        // output position (chunk-local partition index or list position) of the lane's best
  uint32_t n_fit = 0;           // wave-uniform count of partitions that pass the memory filter

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t q_head = 0, q_tail = 0;        // wave-uniform: entries [q_head, q_tail) of the wave's ring wait
  // bounded search: the lowest cost evaluated so far, by this wave or (as of its last look) by any other
  const bool bounded = MODE == 2 && a.s.incumbent != nullptr;
  uint64_t incumbent = ~0ull;
  uint32_t n_eval = 0;                    // wave-uniform count of partitions whose recurrences were run
  if (bounded) incumbent = umin64(a.s.incumbent0, __hip_atomic_load(a.s.incumbent, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  // Bounded search, a whole run at once.  Consecutive ranks differ in their lowest cuts.  When the run of a lane
  // stays inside the block of ranks that share the cuts above the h lowest ones (its offset among the
  // arrangements of those h cuts, plus its length, does not exceed their number C(c[h+1]-1, h)), the stages
  // from h+1 on are the same for every partition of the run, and so is their part of the lower bound: stage s
  // contributes M x its time + the time of all layers ahead of it, whatever the lower cuts are.  If that
  // alone lies above the incumbent for every lane, the wave has nothing to look at.
  bool wave_dead = false;
  if (bounded && K >= 2) {
    uint64_t offset = 0;
    int first_fixed = SP;                   // stages first_fixed.. are the same throughout the run
#pragma unroll
    for (int h = 1; h < K; ++h) {
      offset += BN[(h - 1) * DEV_MAX_L + (c[h] - 1)];
      const bool stays = offset + run_len <= BN[(h - 1) * DEV_MAX_L + (c[h + 1] - 1)];
      first_fixed = (first_fixed == SP && stays) ? h + 1 : first_fixed;
    }
    int pc[SP + 1];                         // forward + backward time of the layers ahead of stage s
#pragma unroll
    for (int s2 = 1; s2 <= SP; ++s2) { const int4 t = T[c[s2]]; pc[s2] = t.x + t.y; }
    int lb = ff->fixed_step;
    for (int ci = 0; ci < ff->n_cls; ++ci) {
      const ClsPtr cl = &ff->cls[ci];
      int v = 0;
#pragma unroll
      for (int s2 = 1; s2 < SP; ++s2) {
        int vs;
        if (STRAT == 0) {
          // a node's own stage and its successor's; the pair that wraps around to stage 0 is left out
          const int pair = s2 + 2 <= SP ? pc[s2 + 2 <= SP ? s2 + 2 : SP] - pc[s2] : 0;
          vs = (s2 == cl->dead0 || s2 == cl->dead1) ? 0 : cl->M * pair;
        } else {
          const int own = pc[s2 + 1] - pc[s2];
          vs = ff->lb_prefix ? (int)__umul24((uint32_t)cl->M, (uint32_t)own) + pc[s2] : cl->M * own;
        }
        v = imax32(v, s2 >= first_fixed ? vs : 0);
      }
      lb = imax32(lb, imax32(0, scale_floor(v, cl->q_min) - cl->lb_slack) + cl->comm_total);
    }
    const uint64_t lb_cost = (uint64_t)scn->K * (uint32_t)lb + (uint64_t)scn->reconf[STRAT];
    const bool look = run_len != 0 && !(first_fixed < SP && lb_cost > incumbent);
    wave_dead = __builtin_amdgcn_ballot_w64(look) == 0;
  }
  // evaluation cuts: the lane's own cuts, or (QUEUED) those of the entry it takes from the ring
  int ce[SP + 1];
  ce[0] = 0;
  ce[SP] = L;

  for (uint32_t it = 0; it < (wave_dead ? 0u : a.per_lane + (QUEUED ? 1u : 0u)); ++it) {
    bool live = it < run_len;             // this lane has a partition in this round
    uint32_t pos = run_first + it;        // where its result is reported
    if (QUEUED) {
      if (it < a.per_lane) {              // uniform; the extra round only drains the ring
        // ---- filter the lane's next partition and append it to the ring if it fits
        int ms[SP], as[SP], cs[SP];           // cs: forward + backward time per stage
        {
          int lo_m = 0, lo_a = 0, lo_c = 0;
#pragma unroll
          for (int j = 0; j < SP; ++j) {
            const int4 hi = T[c[j + 1]];
            ms[j] = hi.z - lo_m;
            as[j] = hi.w - lo_a;
            cs[j] = hi.x + hi.y - lo_c;
            lo_m = hi.z;
            lo_a = hi.w;
            lo_c = hi.x + hi.y;
          }
        }
        bool fits = live && largest_peak<SP, STRAT>(ff, ms, as) <= cap;
        const uint64_t in_memory = __builtin_amdgcn_ballot_w64(fits);
        n_fit += (uint32_t)__popcll(in_memory);
        if (bounded && in_memory != 0) {      // uniform; nothing to bound where nothing fits
          const uint64_t lb_cost = cost_lower_bound<SP, STRAT>(scn, tab, ff, cs, c);
          fits = fits && lb_cost <= incumbent;
        }
        const uint64_t fit_mask = __builtin_amdgcn_ballot_w64(fits);
        if (fits) {
          const uint32_t slot = (uint32_t)wave * QCAP + ((q_tail + (uint32_t)__popcll(fit_mask & ((1ull << lane) - 1ull))) & (QCAP - 1));
          uint32_t words[4] = {0, 0, 0, 0};
#pragma unroll
          for (int i = 1; i <= K; ++i) words[(i - 1) >> 2] |= (uint32_t)c[i] << (8 * ((i - 1) & 3));
          q_cuts[slot] = make_uint4(words[0], words[1], words[2], words[3]);
          q_pos[slot] = (uint32_t)pos;
        }
        q_tail += (uint32_t)__popcll(fit_mask);
        // next partition of the run
        bool done = false;
#pragma unroll
        for (int i = 1; i <= K; ++i) {
          const bool can = c[i] + 1 < c[i + 1];
          c[i] = done ? c[i] : (can ? c[i] + 1 : i);
          done = done || can;
        }
      }
      const uint32_t waiting = q_tail - q_head;
      if (waiting < 64 && !(it == a.per_lane && waiting > 0)) continue;     // uniform
      // ---- evaluate up to 64 waiting entries, one per lane
      const uint32_t take = waiting < 64 ? waiting : 64u;
      live = (uint32_t)lane < take;
      const uint32_t slot = (uint32_t)wave * QCAP + ((q_head + (uint32_t)lane) & (QCAP - 1));
      // lanes past the end take the first partition (cuts 1..K): always valid
      const uint4 packed = live ? q_cuts[slot] : make_uint4(0x04030201u, 0x08070605u, 0x0c0b0a09u, 0x000f0e0du);
      const uint32_t words[4] = {packed.x, packed.y, packed.z, packed.w};
#pragma unroll
      for (int i = 1; i <= K; ++i) ce[i] = (int)((words[(i - 1) >> 2] >> (8 * ((i - 1) & 3))) & 0xffu);
      pos = live ? q_pos[slot] : 0;
      q_head += take;
    }
    if (compact) {
      if (it * BLOCK >= n_slots) break;   // uniform: the region is used up
      const uint32_t slot = it * BLOCK + threadIdx.x;
      live = slot < n_slots;
      // lanes past the end take the first partition (cuts 1..K): always valid
      const uint4 packed = live ? a.cut_list[region + slot] : make_uint4(0x04030201u, 0x08070605u, 0x0c0b0a09u, 0x000f0e0du);
      const uint32_t words[4] = {packed.x, packed.y, packed.z, packed.w};
#pragma unroll
      for (int i = 1; i <= K; ++i) c[i] = (int)((words[(i - 1) >> 2] >> (8 * ((i - 1) & 3))) & 0xffu);
      pos = live ? a.cut_pos[region + slot] : 0;
    }
    if (!QUEUED) {
#pragma unroll
      for (int i = 1; i <= K; ++i) ce[i] = c[i];
    }
    // ---- stage sums from the LDS prefix table
    int fs[SP], bs[SP], ms[SP], as[SP];
    {
      int4 lo = make_int4(0, 0, 0, 0);
#pragma unroll
      for (int j = 0; j < SP; ++j) {
        const int4 hi = T[ce[j + 1]];
        fs[j] = hi.x - lo.x;
        bs[j] = hi.y - lo.y;
        ms[j] = hi.z - lo.z;
        as[j] = hi.w - lo.w;
        lo = hi;
      }
    }
    // ---- memory filter
    // (QUEUED: every entry of the ring has passed it already)
    const bool ok = QUEUED ? live : ((largest_peak<SP, STRAT>(ff, ms, as) <= cap) && live && listed_ok);
    uint64_t cost = (uint64_t)CHM_INF_COST;
    const uint64_t ok_mask = __builtin_amdgcn_ballot_w64(ok);
    if (!QUEUED) n_fit += (uint32_t)__popcll(ok_mask);
    if (ok_mask != 0) {
      int t_step = ff->fixed_step;
      int missing = 0;
      if (STRAT != 1) {
        // weights the stage-j node must fetch: stage size minus what it already holds; prefix
        // sums are monotone, so the prefix at max(a,a0) is the max of the two prefixes
        int have = 0;
        int wl = 0;                      // memory prefix at c[j]
#pragma unroll
        for (int j = 0; j < SP; ++j) {
          const int wh = wl + ms[j];
          have += imax32(0, imin32(wh, ff->w0[j + 1]) - imax32(wl, ff->w0[j]));
          wl = wh;
        }
        missing = ff->w_total - have;
      }
      if (STRAT == 0) {
        int fd[SP], bd[SP];
#pragma unroll
        for (int j = 0; j < SP; ++j) {
          fd[j] = fs[j] + fs[(j + 1) % SP];
          bd[j] = bs[j] + bs[(j + 1) % SP];
        }
        for (int ci = 0; ci < ff->n_cls; ++ci) {
          const ClsPtr cl = &ff->cls[ci];
          int T_c;
          if (cl->n == SP) {
            int F[SP], B[SP];
#pragma unroll
            for (int j = 0; j < SP; ++j) { F[j] = fd[j]; B[j] = bd[j]; }
            T_c = class_time<SP>(cl, F, B);
          } else if (SP >= 2 && cl->n == SP - 1) {
            constexpr int N = SP >= 2 ? SP - 1 : 1;
            int F[N], B[N];
#pragma unroll
            for (int j = 0; j < N; ++j) {
              const bool before = j < cl->dead0;
              F[j] = before ? fd[j] : fd[(j + 1) % SP];
              B[j] = before ? bd[j] : bd[(j + 1) % SP];
            }
            T_c = class_time<N>(cl, F, B);
          } else {
            constexpr int N = SP >= 3 ? SP - 2 : 1;
            int F[N], B[N];
#pragma unroll
            for (int j = 0; j < N; ++j) {
              const bool b0 = j < cl->dead0, b1 = j + 1 < cl->dead1;
              F[j] = b0 ? fd[j] : (b1 ? fd[(j + 1) % SP] : fd[(j + 2) % SP]);
              B[j] = b0 ? bd[j] : (b1 ? bd[(j + 1) % SP] : bd[(j + 2) % SP]);
            }
            T_c = class_time<N>(cl, F, B);
          }
          t_step = imax32(t_step, T_c);
        }
      } else {
        for (int ci = 0; ci < ff->n_cls; ++ci) {
          const ClsPtr cl = &ff->cls[ci];
          int F[SP], B[SP];
#pragma unroll
          for (int j = 0; j < SP; ++j) { F[j] = fs[j]; B[j] = bs[j]; }
          t_step = imax32(t_step, class_time<SP>(cl, F, B));
          if (STRAT == 1) {
            int have = 0;
            if (ff->assign) {
              // least-transfer assignment = largest total overlap of a non-crossing matching of survivors
              // and new stages (both are in layer order, see best_overlap in chm_kernels.hip); one row of
              // the two-index recurrence lives in registers.  A negative raw overlap needs no clamp:
              // diag + (negative) < diag <= G[j], which is already among the operands of the max.
              int G[SP + 1];
#pragma unroll
              for (int j = 0; j <= SP; ++j) G[j] = 0;
#pragma unroll
              for (int i = 0; i < SP; ++i) {
                const int wlo_i = cl->wlo[i], whi_i = cl->whi[i];
                int diag = 0, wl = 0;
#pragma unroll
                for (int j = 0; j < SP; ++j) {
                  const int wh = wl + ms[j];
                  const int above = G[j + 1];
                  const int cand = diag + (imin32(wh, whi_i) - imax32(wl, wlo_i));
                  G[j + 1] = imax32(imax32(above, G[j]), cand);
                  diag = above;
                  wl = wh;
                }
              }
              have = G[SP];
            } else {
              int wl = 0;
#pragma unroll
              for (int j = 0; j < SP; ++j) {
                const int wh = wl + ms[j];
                have += imax32(0, imin32(wh, cl->whi[j]) - imax32(wl, cl->wlo[j]));
                wl = wh;
              }
            }
            missing = imax32(missing, ff->w_total - have);
          }
        }
      }
      if (ff->allreduce > 0) {
        // rounds of gradient communication: largest stage on any device, or the ring colouring when nodes hold two stages
        int rounds;
        if (STRAT == 0) {
          rounds = ring_rounds<SP>(ce, ff->node_exists);
        } else {
          rounds = ff->fixed_layers;
#pragma unroll
          for (int j = 0; j < SP; ++j) rounds = imax32(rounds, ce[j + 1] - ce[j]);
        }
        t_step += ff->allreduce * rounds;
      }
      if (STRAT == 2 && (QUEUED || a.base_out == nullptr)) {
        // every reroute vector of every stage that lost nodes
        for (int st = 0; st < scn->n_aff; ++st) {
          const int sa = scn->aff_stage[st];
          int f_st = fs[0], b_st = bs[0];
#pragma unroll
          for (int j = 1; j < SP; ++j) {
            f_st = sa == j ? fs[j] : f_st;
            b_st = sa == j ? bs[j] : b_st;
          }
          const int p = scn->aff_peers[st];
          const RowPtr runs = as_const(a.runs) + tab->run_off[st];
          const uint32_t n_runs = tab->run_count[st];
          uint32_t pen = 0;
          if (QUEUED && a.capacity_penalty) {
            // reroute spaces too large to sweep here (a bounded search does not use the sweep kernels)
            uint32_t w[FAST_MAX_P];
#pragma unroll
            for (int i = 0; i < FAST_MAX_P; ++i) w[i] = i < p ? peer_time(f_st, b_st, scn->aff_q[st][i < p ? i : 0]) : 0u;
            const uint32_t orphans = (uint32_t)scn->aff_total[st];
            pen = least_penalty32(w, p, orphans, scn->rcap > 0 ? (uint32_t)scn->rcap : orphans);
            t_step += (int)pen;
            continue;
          }
          const uint32_t shape = tab->unrolled_shape[st];
          if (shape != 0) {
            // small uncapped spaces: sweep unrolled at compile time over a table of products
#define CHM_UNROLLED(P, T)                                                                      \
  case (P) * 256 + (T): {                                                                       \
    uint32_t w[P];                                                                              \
    _Pragma("unroll") for (int i = 0; i < P; ++i) {                                             \
      const uint32_t q = scn->aff_q[st][i];                                                     \
      w[i] = peer_time(f_st, b_st, q);                                                          \
    }                                                                                           \
    pen = sweep_products<P, T>(w);                                                              \
  } break;
            switch (shape) {
              CHM_UNROLLED(2, 8) CHM_UNROLLED(2, 16) CHM_UNROLLED(2, 32)
              CHM_UNROLLED(3, 8) CHM_UNROLLED(3, 16)
              default: break;
            }
#undef CHM_UNROLLED
            t_step += (int)pen;
            continue;
          }
#define CHM_SWEEP(P)                                                                            \
  case P: {                                                                                     \
    uint32_t w[P];                                                                              \
    _Pragma("unroll") for (int i = 0; i < P; ++i) {                                             \
      const uint32_t q = scn->aff_q[st][i];                                                     \
      w[i] = peer_time(f_st, b_st, q);                                                          \
    }                                                                                           \
    pen = sweep_runs<P>(runs, n_runs, w);                                                       \
  } break;
          switch (p) {
            CHM_SWEEP(1) CHM_SWEEP(2) CHM_SWEEP(3) CHM_SWEEP(4)
            CHM_SWEEP(5) CHM_SWEEP(6) CHM_SWEEP(7) CHM_SWEEP(8)
            default: break;
          }
#undef CHM_SWEEP
          t_step += (int)pen;
        }
      }
      if (!QUEUED && STRAT == 2 && a.base_out != nullptr) {
        // split path: hand the peer stage times of this partition to the sweep kernel
        if (ok) {
          uint32_t *wout = a.weights_out + (size_t)(run_first + it) * (DEV_MAX_AFF * 8);
          for (int st = 0; st < scn->n_aff; ++st) {
            const int sa = scn->aff_stage[st];
            int f_st = fs[0], b_st = bs[0];
#pragma unroll
            for (int j = 1; j < SP; ++j) {
              f_st = sa == j ? fs[j] : f_st;
              b_st = sa == j ? bs[j] : b_st;
            }
            const int p = scn->aff_peers[st];
            for (int i = 0; i < p; ++i) {
              const uint32_t q = scn->aff_q[st][i];
              wout[st * 8 + i] = peer_time(f_st, b_st, q);
            }
          }
        }
      }
      cost = (uint64_t)scn->K * (uint32_t)t_step + (uint64_t)scn->reconf[STRAT] + (uint64_t)scn->xfer * (uint32_t)missing;
      // a lane meets the entries of a compacted list or of a ring in no particular order of position:
      // there the lower position wins among equal costs; a run is walked in ascending order
      const bool lower = (QUEUED || compact) ? (cost < best_cost || (cost == best_cost && pos < best_pos)) : cost < best_cost;
      if (ok && lower) { best_cost = cost; best_pos = pos; }
      if (bounded) {
        // the round's lowest cost becomes known to every wave; what the others found is picked up in turn
        n_eval += (uint32_t)__popcll(ok_mask);
        const uint64_t round_best = wave_min(ok ? cost : ~0ull);
        if (round_best < incumbent) {
          incumbent = round_best;
          if (lane == 0) atomicMin((unsigned long long *)a.s.incumbent, (unsigned long long)round_best);
        }
        incumbent = umin64(incumbent, __hip_atomic_load(a.s.incumbent, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
      }
      if (!QUEUED && STRAT == 2 && a.base_out != nullptr && ok) a.base_out[run_first + it] = cost;
    }
    if (!QUEUED && STRAT == 2 && a.base_out != nullptr && !ok && it < run_len) a.base_out[run_first + it] = ~0ull;
    if (!QUEUED && a.s.costs_out != nullptr) {
      // per_lane == 1: the store is coalesced as it is; longer runs go through an LDS tile
      // (laid out in output order) and are written out together after the loop
      const int64_t v = ok ? (int64_t)cost : CHM_INF_COST;
      if (a.per_lane == 1 || compact) { if (live) a.s.costs_out[pos] = v; }
      else cost_tile[threadIdx.x * a.per_lane + it] = v;
    }
    // ---- next partition in rank order: bump the lowest cut that has room, reset those below
    if (!compact && !QUEUED) {
      bool done = false;
#pragma unroll
      for (int i = 1; i <= K; ++i) {
        const bool can = c[i] + 1 < c[i + 1];
        c[i] = done ? c[i] : (can ? c[i] + 1 : i);
        done = done || can;
      }
    }
  }

  if (!QUEUED && a.s.costs_out != nullptr && a.per_lane > 1 && !compact) {
    __syncthreads();
    const uint64_t block_first = (uint64_t)blockIdx.x * BLOCK * a.per_lane;
    const uint32_t n_tile = BLOCK * a.per_lane;
    for (uint32_t i = threadIdx.x; i < n_tile; i += BLOCK)
      if (block_first + i < a.s.part_count) a.s.costs_out[block_first + i] = cost_tile[i];
  }
  uint64_t key = best_cost == ~0ull ? CHM_KEY_NONE
                                    : ((best_cost << a.s.idx_bits) | (uint64_t)best_pos);
  if (!QUEUED && STRAT == 2 && a.base_out != nullptr) key = CHM_KEY_NONE;   // the combine kernel takes the argmin
  key = wave_min(key);
  if (lane == 0) { wave_keys[wave] = key; wave_fit[wave] = n_fit; wave_eval[wave] = n_eval; }
  __syncthreads();
  if (threadIdx.x == 0) {
    // one atomic of each kind per workgroup, spread over several words (see SearchLaunch)
    const uint32_t slot = (blockIdx.x & a.s.slot_mask) * a.s.slot_stride;
    uint64_t k = wave_keys[0];
    uint32_t fit = wave_fit[0], evaluated = wave_eval[0];
#pragma unroll
    for (int i = 1; i < BLOCK / 64; ++i) { k = umin64(k, wave_keys[i]); fit += wave_fit[i]; evaluated += wave_eval[i]; }
    if (fit) atomicAdd((unsigned long long *)a.s.feasible + slot, (unsigned long long)fit);
    if (bounded && evaluated) atomicAdd((unsigned long long *)a.s.evaluated + slot, (unsigned long long)evaluated);
    // a search over a list of candidates of a bounded search makes its best cost known to what follows
    if (!QUEUED && a.s.incumbent != nullptr && k != CHM_KEY_NONE)
      atomicMin((unsigned long long *)a.s.incumbent, (unsigned long long)(k >> a.s.idx_bits));
    if (k != CHM_KEY_NONE) atomicMin((unsigned long long *)a.s.result + slot, (unsigned long long)k);
  }
}

// ---------------------------------------------------------------------------------------
// explicit lists: memory filter and compaction
// ---------------------------------------------------------------------------------------
// One lane per list entry: cut positions (given, or unranked), stage memory sums, memory filter.  An entry
// that does not fit (or is malformed) gets its cost (infeasible) right away; the others are appended to the
// workgroup's own region of a compact list as (cut positions packed into 16 bytes, list position).  Slots are
// handed out through a counter in LDS: atomics of many workgroups on one global counter would serialise (about
// 10 ns each).  The search kernel then runs over every region with all lanes busy.
constexpr int FILTER_TILES = 16;        // tiles of BLOCK entries per workgroup = rounds of the search kernel per region
constexpr int FILTER_TILES_BOUNDED = 4;  // a bounded search keeps few entries: shorter regions, more workgroups to filter with

struct ListFilter {
  const DevScenario *scn;
  const FastTables *tab;
  const uint64_t *ranks;        // list entries of this pass, as partition ranks, or (ranks null)
  const uint8_t *cuts;          // as rows of stages - 1 cut positions
  uint32_t n;                   // entries in this pass
  uint32_t pos_base;            // list position (chunk-local) of entry 0 of this pass
  int64_t *costs_out;           // chunk-local cost array (nullable)
  int32_t tiles;                // tiles of BLOCK entries per workgroup
  uint4 *cut_list;              // [workgroup][tiles * BLOCK]
  uint32_t *cut_pos;            // likewise
  uint32_t *cut_count;          // [workgroup] filled slots
  // bounded search (no cost store): entries whose lower bound of the cost lies above *incumbent (the lowest cost
  // the passes before this one have evaluated) are dropped like those that do not fit; null = keep all that fit
  const uint64_t *incumbent;
  uint64_t incumbent0;          // a cost known before the call (see SearchLaunch::incumbent0)
};

template <int SP, int STRAT>
__global__ void __launch_bounds__(BLOCK) k_list_filter(ListFilter a) {
  constexpr int K = SP - 1;
  __shared__ int4 T[DEV_MAX_L + 1];
  __shared__ uint64_t BN[(K > 0 ? K : 1) * DEV_MAX_L];
  __shared__ uint32_t filled;
  const ScnPtr scn = as_const(a.scn);
  const TabPtr tab = as_const(a.tab);
  const FamPtr ff = &tab->fam[STRAT];
  const int L = scn->L;
  const bool bounded = a.incumbent != nullptr && a.costs_out == nullptr;
  const uint64_t incumbent = bounded ? umin64(a.incumbent0, __hip_atomic_load(a.incumbent, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) : ~0ull;
  for (int i = threadIdx.x; i <= L; i += BLOCK) T[i] = make_int4((int)scn->pf[i], (int)scn->pb[i], (int)scn->pw[i], (int)scn->pa[i]);
  if (a.cuts == nullptr)
    for (int i = threadIdx.x; i < K * DEV_MAX_L; i += BLOCK) BN[i] = scn->binom[1 + i / DEV_MAX_L][i % DEV_MAX_L];
  if (threadIdx.x == 0) filled = 0;
  __syncthreads();
  const uint32_t region = blockIdx.x * ((uint32_t)a.tiles * BLOCK);
  for (int tile = 0; tile < a.tiles; ++tile) {
    const uint32_t gid = region + tile * BLOCK + threadIdx.x;
    if (gid - threadIdx.x >= a.n) break;                        // uniform: this tile and the next ones are empty
    const bool live = gid < a.n;
    int c[SP + 1];
    c[0] = 0;
    c[SP] = L;
    bool valid = live;
    if (a.cuts != nullptr) {
      // explicit cut positions; a row that does not increase strictly within 1..L-1 is replaced by 1..K
      const uint8_t *row = a.cuts + (size_t)(live ? gid : 0) * K;
      int prev = 0;
#pragma unroll
      for (int i = 1; i <= K; ++i) {
        c[i] = row[i - 1];
        valid = valid && c[i] > prev && c[i] <= L - 1;
        prev = c[i];
      }
      if (!valid) {
#pragma unroll
        for (int i = 1; i <= K; ++i) c[i] = i;
      }
    } else {
      uint64_t rem = live ? a.ranks[gid] : 0;
      valid = live && rem < scn->fam[STRAT].n_part;
      if (!valid) rem = 0;
      unrank_digits<K>(rem, L, (L - 1) <= 64 ? 3 : 4, BN, c);
    }
    int ms[SP], as[SP], cs[SP];
    {
      int lo_m = 0, lo_a = 0, lo_c = 0;
#pragma unroll
      for (int j = 0; j < SP; ++j) {
        const int4 hi = T[c[j + 1]];
        ms[j] = hi.z - lo_m;
        as[j] = hi.w - lo_a;
        cs[j] = hi.x + hi.y - lo_c;
        lo_m = hi.z;
        lo_a = hi.w;
        lo_c = hi.x + hi.y;
      }
    }
    bool ok = valid && largest_peak<SP, STRAT>(ff, ms, as) <= (int)scn->cap;
    if (bounded && incumbent != ~0ull && __builtin_amdgcn_ballot_w64(ok) != 0)      // uniform
      ok = ok && cost_lower_bound<SP, STRAT>(scn, tab, ff, cs, c) <= incumbent;
    if (live && !ok && a.costs_out != nullptr) a.costs_out[a.pos_base + gid] = CHM_INF_COST;
    const uint64_t mask = __builtin_amdgcn_ballot_w64(ok);
    if (mask != 0) {
      const int lane = threadIdx.x & 63;
      uint32_t base = 0;
      if (lane == 0) base = atomicAdd(&filled, (uint32_t)__popcll(mask));
      base = __shfl(base, 0, 64);
      if (ok) {
        const uint32_t slot = region + base + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
        uint32_t words[4] = {0, 0, 0, 0};
#pragma unroll
        for (int i = 1; i <= K; ++i) words[(i - 1) >> 2] |= (uint32_t)c[i] << (8 * ((i - 1) & 3));
        a.cut_list[slot] = make_uint4(words[0], words[1], words[2], words[3]);
        a.cut_pos[slot] = a.pos_base + gid;
      }
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) a.cut_count[blockIdx.x] = filled;
}

// ---------------------------------------------------------------------------------------
// bounded search: enumeration of the candidates (see CandidateSet)
// ---------------------------------------------------------------------------------------
// row[x] = candidates (of the arrangement being refined) whose current stage starts at or before x.  Finds by
// bisection the start in [lo, hi] whose block holds index idx, counting blocks from lo on, and leaves in idx
// the offset inside that block (an index beyond the last block lands on hi).
__host__ __device__ inline int candidate_start(const uint64_t *row, int lo, int hi, uint64_t &idx) {
  const uint64_t target = idx + (lo > 0 ? row[lo - 1] : 0);
  int a = lo, b = hi;
  while (a < b) {
    const int m = (a + b) >> 1;
    if (row[m] > target) b = m;
    else a = m + 1;
  }
  idx = target - (a > 0 ? row[a - 1] : 0);
  return a;
}

struct CandidateEnum {
  const uint64_t *ways;         // [stages][end][start]
  const uint8_t *low_pair;      // [stages][L+1]
  int32_t stages, L;
  uint32_t total;               // candidates of this launch
  uint64_t first, stride;       // launch index i stands for candidate (first + i) * stride
  uint4 *cut_list;              // [candidate] cut positions packed into bytes
  uint32_t *cut_pos;            // [candidate] = its index
  uint32_t *cut_count;          // [workgroup] candidates in its region of BLOCK slots
};

// Candidate `index` of the set, in ascending partition rank: the start of the last stage is chosen first
// (the candidates that share it form a block of ways[last][a][L] indices), then the start of the stage below
// it among those the pair limit allows, and so on down.  Every scan is bounded by the stage above it, so the
// cuts stay a valid partition whatever the tables hold.
__global__ void __launch_bounds__(BLOCK) k_enumerate_candidates(CandidateEnum e) {
  const uint32_t gid = blockIdx.x * BLOCK + threadIdx.x;
  if (threadIdx.x == 0) {
    const uint32_t first = blockIdx.x * BLOCK;
    e.cut_count[blockIdx.x] = first >= e.total ? 0u : (e.total - first < BLOCK ? e.total - first : (uint32_t)BLOCK);
  }
  if (gid >= e.total) return;
  const int W = e.L + 1;
  uint64_t idx = (e.first + gid) * e.stride;
  uint32_t words[4] = {0, 0, 0, 0};
  int s = e.stages - 1;                   // the stage whose start is being chosen
  int end = e.L;                          // its end
  // at least one layer for every stage below
  int start = candidate_start(e.ways + ((size_t)s * W + end) * W, s, end - 1, idx);
  for (;;) {
    words[(s - 1) >> 2] |= (uint32_t)start << (8 * ((s - 1) & 3));
    if (s == 1) break;
    // the stage below: layers [below, start), its pair with stage s ends at `end`
    const int lo = (int)e.low_pair[(size_t)(s - 1) * W + end];
    const int first = lo > s - 1 ? lo : s - 1;
    const int below = first >= start - 1 ? start - 1 : candidate_start(e.ways + ((size_t)(s - 1) * W + start) * W, first, start - 1, idx);
    end = start;
    start = below;
    --s;
  }
  e.cut_list[gid] = make_uint4(words[0], words[1], words[2], words[3]);
  e.cut_pos[gid] = gid;
}

// ---------------------------------------------------------------------------------------
// reroute vector table and the split rerouting path
// ---------------------------------------------------------------------------------------
// Row r of affected stage a = the reroute vector of rank r, decoded from the count table
// (count[left][remaining] = vectors of `left` entries summing to `remaining`); rows beyond the
// valid ones put every orphaned micro-batch on every peer (never better than a valid row).
__global__ void __launch_bounds__(BLOCK) k_make_rows(const DevScenario *__restrict__ scn, const uint64_t *__restrict__ comp,
                                                     int a, uint32_t *__restrict__ rows, uint32_t n_rows_padded, int stride) {
  const uint32_t r = blockIdx.x * BLOCK + threadIdx.x;
  if (r >= n_rows_padded) return;
  const int p = scn->aff_peers[a];
  const int total = scn->aff_total[a];
  uint32_t *row = rows + (size_t)r * stride;
  if ((uint64_t)r >= scn->aff_R[a]) {
    for (int i = 0; i < stride; ++i) row[i] = i < p ? (uint32_t)total : 0u;
    return;
  }
  const uint64_t *tab = comp + scn->comp_off[a];
  const uint32_t cs = scn->comp_stride[a];
  uint64_t rank = r;
  int rem = total;
  for (int pos = 0; pos < stride; ++pos) {
    int v = 0;
    if (pos < p) {
      const int left = p - 1 - pos;
      for (;; ++v) {
        const uint64_t cnt = tab[(uint32_t)left * cs + (uint32_t)(rem - v)];
        if (rank < cnt) break;
        rank -= cnt;
      }
      rem -= v;
    }
    row[pos] = (uint32_t)v;
  }
}

// best penalty of one affected stage for 256 partitions (one per lane) over one chunk of runs
template <int P>
__global__ void __launch_bounds__(BLOCK) k_sweep(const uint32_t *__restrict__ runs, uint32_t n_runs, uint32_t runs_per_chunk,
                                                 const uint64_t *__restrict__ base, const uint32_t *__restrict__ weights,
                                                 uint32_t *__restrict__ pen_best, uint32_t part_count, int a) {
  const uint32_t part = blockIdx.x * BLOCK + threadIdx.x;
  const bool live = part < part_count && base[part < part_count ? part : 0] != ~0ull;
  if (__builtin_amdgcn_ballot_w64(live) == 0) return;       // a wave of partitions that do not fit
  uint32_t w[P];
#pragma unroll
  for (int i = 0; i < P; ++i) w[i] = live ? weights[(size_t)part * (DEV_MAX_AFF * 8) + a * 8 + i] : 1u;
  const uint32_t first = blockIdx.y * runs_per_chunk;
  const uint32_t n = first >= n_runs ? 0u : (n_runs - first < runs_per_chunk ? n_runs - first : runs_per_chunk);
  const uint32_t pen = sweep_runs<P>(as_const(runs) + (size_t)first * 8, n, w);
  if (live && n) atomicMin(&pen_best[(size_t)part * DEV_MAX_AFF + a], pen);
}

// The partitions of a pass that fit in memory (base cost known), gathered into a list so that the sweep kernels
// keep every lane busy; the order within the list is of no consequence (results go back by partition).
__global__ void __launch_bounds__(BLOCK) k_compact_fit(const uint64_t *__restrict__ base, uint32_t part_count,
                                                       uint32_t *__restrict__ list, uint32_t *__restrict__ count) {
  const uint32_t part = blockIdx.x * BLOCK + threadIdx.x;
  const bool fit = part < part_count && base[part < part_count ? part : 0] != ~0ull;
  const uint64_t mask = __builtin_amdgcn_ballot_w64(fit);
  if (mask == 0) return;
  const int lane = threadIdx.x & 63;
  uint32_t first = 0;
  if (lane == 0) first = atomicAdd(count, (uint32_t)__popcll(mask));
  first = __shfl(first, 0, 64);
  if (fit) list[first + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull))] = part;
}

// min over the pairs (a, b) with a + b = REM, 0 <= a, b <= CAP of max(A[a], B[b]): the last two entries of a reroute
// vector, their products read from register tables at compile-time positions (one v_max_u32 and half a v_min3_u32
// per vector)
template <int REM, int CAP>
__device__ __forceinline__ uint32_t pair_min(const uint32_t (&A)[CAP + 1], const uint32_t (&B)[CAP + 1]) {
  constexpr int LO = REM > CAP ? REM - CAP : 0, HI = REM < CAP ? REM : CAP;
  uint32_t m = 0xffffffffu;
#pragma unroll
  for (int a = LO; a <= HI; ++a) {
    const uint32_t z = A[a] > B[REM - a] ? A[a] : B[REM - a];
    m = m < z ? m : z;
  }
  return m;
}

// pair_min for every remaining sum REM..0, stored to the lane's column of an LDS table
template <int REM, int CAP>
__device__ __forceinline__ void pair_minima(const uint32_t (&A)[CAP + 1], const uint32_t (&B)[CAP + 1], uint32_t (*table)[BLOCK], int tid) {
  table[REM][tid] = pair_min<REM, CAP>(A, B);
  if constexpr (REM > 0) pair_minima<REM - 1, CAP>(A, B, table, tid);
}

// Best penalty of one affected stage for the partitions of the fit list (one per lane) over one chunk of groups.
// The penalty of a reroute vector is the largest of its P products (extra micro-batches x peer stage time).  The
// vectors of a group share their first P-3 entries, whose largest product is taken once per group.  The entry
// before the last two steps through consecutive values (its product is carried by an add); for each of its values
// the last two entries run over all pairs with the remaining sum, and the least of the larger of their two
// products depends on that sum alone: the 2*CAP+1 such minima are worked out once per lane (every pair scored
// once, products from two register tables r x peer time, r = 0..CAP) and kept in the lane's column of an LDS
// table.  A value of the stepping entry then costs one LDS read, one v_max3_u32, one v_min_u32 and one add for
// all vectors that share it.  All control flow is uniform (descriptors come through scalar loads).
template <int P, int CAP>
__global__ void __launch_bounds__(BLOCK) k_sweep_groups(const uint32_t *__restrict__ groups, uint32_t n_groups, uint32_t groups_per_chunk,
                                                        const uint32_t *__restrict__ fit_list, const uint32_t *__restrict__ fit_count,
                                                        const uint32_t *__restrict__ weights, uint32_t *__restrict__ pen_best, int a) {
  static_assert(P >= 3 && P <= 8 && (CAP == 8 || CAP == 16), "three to eight peers, entries up to 8 or 16");
  constexpr int Q = P - 3;                            // shared entries per group
  __shared__ uint32_t pairs[2 * CAP + 1][BLOCK];      // [remaining sum][lane]: read and written by its own lane only
  const uint32_t n_fit = *as_const(fit_count);
  if (blockIdx.x * BLOCK >= n_fit) return;            // uniform: this block has no partition
  const int tid = threadIdx.x;
  const uint32_t slot = blockIdx.x * BLOCK + threadIdx.x;
  const bool live = slot < n_fit;
  const uint32_t part = fit_list[live ? slot : n_fit - 1];    // lanes past the end redo the last partition
  uint32_t w[P];
#pragma unroll
  for (int i = 0; i < P; ++i) w[i] = weights[(size_t)part * (DEV_MAX_AFF * 8) + a * 8 + i];
  const uint32_t first = blockIdx.y * groups_per_chunk;
  const uint32_t n = first >= n_groups ? 0u : (n_groups - first < groups_per_chunk ? n_groups - first : groups_per_chunk);
  if (n == 0) return;
  {
    uint32_t A[CAP + 1], B[CAP + 1];
    A[0] = 0;
    B[0] = 0;
#pragma unroll
    for (int r = 1; r <= CAP; ++r) { A[r] = A[r - 1] + w[P - 2]; B[r] = B[r - 1] + w[P - 1]; }
    pair_minima<2 * CAP, CAP>(A, B, pairs, tid);
  }
  const uint32_t wv = w[P - 3];
  const RowPtr tab = as_const(groups) + (size_t)first * 8;
  uint32_t best = 0xffffffffu;
  // the descriptor of the next group is fetched while the current one is swept
  uint32_t d[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) d[i] = tab[i];
  for (uint32_t g = 0; g < n; ++g) {
    uint32_t nx[8];
    const RowPtr nd = tab + (size_t)(g + 1 < n ? g + 1 : g) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) nx[i] = nd[i];
    uint32_t pre = 0;
#pragma unroll
    for (int i = 0; i < Q; ++i) {
      const uint32_t v = __umul24(d[i], w[i]);
      pre = pre > v ? pre : v;
    }
    uint32_t pv = __umul24(d[5], wv);                 // product of the stepping entry at its first value
    const uint32_t cnt = d[6];                        // values it takes
    const uint32_t rem2 = d[7] - d[5];                // what the last two entries add up to at its first value (<= 2 * CAP)
#pragma unroll 4
    for (uint32_t r = 0; r < cnt; ++r) {
      const uint32_t m = pairs[rem2 - r][tid];
      uint32_t pen = pre > pv ? pre : pv;
      pen = pen > m ? pen : m;
      best = best < pen ? best : pen;
      pv += wv;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) d[i] = nx[i];
  }
  if (live) atomicMin(&pen_best[(size_t)part * DEV_MAX_AFF + a], best);
}

// The least penalty of one affected stage without looking at the vectors one by one.  A vector r (r_i extra
// micro-batches on peer i, r_i <= cap, sum = orphans) has penalty max_i r_i * w_i <= v exactly when r_i <=
// floor(v / w_i) for every peer, so some vector reaches v iff sum_i min(cap, floor(v / w_i)) >= orphans.  That
// sum grows with v: the least v that satisfies it, found by bisection, is the minimum over all vectors (it is
// one of the products r_i * w_i, since the sum only steps there).  One lane per partition; the winner's
// vectors are recovered afterwards as usual.
__global__ void __launch_bounds__(BLOCK) k_least_penalty(const uint64_t *__restrict__ base, const uint32_t *__restrict__ weights,
                                                         uint32_t *__restrict__ pen_best, uint32_t part_count, int a, int peers,
                                                         uint32_t orphans, uint32_t cap) {
  const uint32_t part = blockIdx.x * BLOCK + threadIdx.x;
  if (part >= part_count || base[part] == ~0ull) return;
  uint32_t w[FAST_MAX_P];
  uint32_t w_max = 1;
#pragma unroll
  for (int i = 0; i < FAST_MAX_P; ++i) {
    w[i] = i < peers ? weights[(size_t)part * (DEV_MAX_AFF * 8) + a * 8 + i] : 0u;
    w_max = w[i] > w_max ? w[i] : w_max;
  }
  uint64_t lo = 0, hi = (uint64_t)orphans * w_max;       // every peer can take all orphans within hi (if the cap lets it)
  while (lo < hi) {
    const uint64_t v = lo + (hi - lo) / 2;
    uint64_t room = 0;
#pragma unroll
    for (int i = 0; i < FAST_MAX_P; ++i) {
      if (i < peers) {
        const uint64_t fit = w[i] == 0 ? (uint64_t)cap : v / w[i];
        room += fit < cap ? fit : (uint64_t)cap;
      }
    }
    if (room >= orphans) hi = v;
    else lo = v + 1;
  }
  pen_best[(size_t)part * DEV_MAX_AFF + a] = (uint32_t)lo;
}

// cost = cost without penalties + K * sum of the per-stage best penalties; argmin as usual
__global__ void __launch_bounds__(BLOCK) k_combine(const uint64_t *__restrict__ base, const uint32_t *__restrict__ pen_best,
                                                   uint32_t part_count, int n_aff, uint64_t K, uint32_t index_base,
                                                   int idx_bits, uint64_t *result) {
  __shared__ uint64_t wave_keys[BLOCK / 64];
  const uint32_t part = blockIdx.x * BLOCK + threadIdx.x;
  uint64_t key = CHM_KEY_NONE;
  if (part < part_count && base[part] != ~0ull) {
    uint64_t pen = 0;
    for (int a = 0; a < n_aff; ++a) pen += pen_best[(size_t)part * DEV_MAX_AFF + a];
    key = ((base[part] + K * pen) << idx_bits) | (uint64_t)(index_base + part);
  }
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

struct ExpandArgs {
  const uint64_t *base;         // [partition of the pass] cost without penalties, ~0 = does not fit
  const uint32_t *weights;      // [partition of the pass][affected stage][8]
  const uint32_t *rows[DEV_MAX_AFF];
  uint64_t R[DEV_MAX_AFF];      // valid reroute vectors per affected stage
  int32_t stride[DEV_MAX_AFF], peers[DEV_MAX_AFF];
  int32_t n_aff;
  uint64_t R_joint, K;
  uint64_t local_first, count;  // plan indices local to the family
  uint64_t part_base;           // first partition of the pass
  int64_t *costs;
};

// one lane per plan index: split the index into (partition, per-stage reroute ranks), look the
// vectors up, add the penalties to the partition's base cost, store (coalesced)
__global__ void __launch_bounds__(BLOCK) k_expand(ExpandArgs a) {
  const uint64_t gid = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
  if (gid >= a.count) return;
  const uint64_t local = a.local_first + gid;
  const uint64_t part = local / a.R_joint;
  uint64_t rr = local - part * a.R_joint;
  const uint64_t pl = part - a.part_base;
  const uint64_t base = a.base[pl];
  uint64_t pen = 0;
  for (int s = a.n_aff - 1; s >= 0; --s) {          // last affected stage is least significant
    const uint64_t q = rr / a.R[s];
    const uint64_t r = rr - q * a.R[s];
    rr = q;
    const uint32_t *row = a.rows[s] + r * (uint64_t)a.stride[s];
    const uint32_t *w = a.weights + pl * (DEV_MAX_AFF * 8) + s * 8;
    uint32_t m = 0;
    for (int i = 0; i < a.peers[s]; ++i) {
      const uint32_t v = base != ~0ull ? __umul24(row[i], w[i]) : 0u;
      m = m > v ? m : v;
    }
    pen += m;
  }
  __builtin_nontemporal_store((int64_t)(base == ~0ull ? CHM_INF_COST : (int64_t)(base + a.K * pen)), &a.costs[gid]);
}

// The same with 32-bit index arithmetic, for reroute spaces below 2^31 vectors per partition and launches
// of at most 2^31 plan indices: the host passes the partition (relative to the pass) and the reroute rank of
// the launch's first plan index, so a lane divides first_rr + gid, which fits 32 bits.
// Division of a 32-bit number by a divisor fixed at launch: one multiply-high, two shifts, an add and a subtract
// (round-up method of Granlund and Montgomery), exact for every dividend; the compiler's generic 32-bit
// division costs about five times as much.
struct FastDiv {
  uint32_t d, m, sh1, sh2;
};
static FastDiv make_fast_div(uint32_t d) {
  FastDiv f;
  f.d = d;
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;                               // ceil(log2 d)
  f.m = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d) + 1u;
  f.sh1 = l < 1 ? l : 1;
  f.sh2 = l > 0 ? l - 1 : 0;
  return f;
}
__device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDiv &f) {
  const uint32_t t = __umulhi(f.m, n);
  return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

struct ExpandArgs32 {
  const uint64_t *base;
  const uint32_t *weights;
  const uint32_t *rows[DEV_MAX_AFF];
  FastDiv R[DEV_MAX_AFF];
  int32_t stride[DEV_MAX_AFF], peers[DEV_MAX_AFF];
  int32_t n_aff;
  FastDiv R_joint;
  uint32_t first_part, first_rr, count;
  uint64_t K;
  int64_t *costs;
};

// Plan indices per workgroup: EXPAND_PER consecutive tiles of BLOCK.  A lane computes its EXPAND_PER costs
// first and stores them back to back at the end: memory operations of a wave complete in order, so a load
// issued after a store would wait for that store to be acknowledged (microseconds when HBM is saturated
// with writes), and with one 512-byte store in flight per wave the kernel stayed below 1.5 TB/s.
constexpr int EXPAND_PER = 8;

__device__ __forceinline__ int64_t expand_one(const ExpandArgs32 &a, uint32_t gid) {
  const uint32_t idx = a.first_rr + gid;
  const uint32_t q = fast_div(idx, a.R_joint);
  uint32_t rr = idx - q * a.R_joint.d;
  const uint32_t pl = a.first_part + q;
  const uint64_t base = a.base[pl];
  uint64_t pen = 0;
  // unrolled over the (at most four) affected stages so that the per-stage launch arguments are read with
  // constant offsets; rows are padded to 4 or 8 entries with zeros, so whole rows are read
#pragma unroll
  for (int s = DEV_MAX_AFF - 1; s >= 0; --s) {      // last affected stage is least significant
    if (s < a.n_aff) {
      uint32_t r = rr;
      if (s > 0) {                                  // the first stage takes what is left: no division
        const uint32_t qq = fast_div(rr, a.R[s]);
        r = rr - qq * a.R[s].d;
        rr = qq;
      }
      const uint32_t *w = a.weights + (size_t)pl * (DEV_MAX_AFF * 8) + s * 8;
      const uint32_t *row = a.rows[s] + (size_t)r * (uint32_t)a.stride[s];
      uint32_t m = 0;
      if (a.stride[s] == 4) {
#pragma unroll
        for (int i = 0; i < 4; ++i) m = max(m, __umul24(row[i], w[i]));
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) m = max(m, __umul24(row[i], w[i]));
      }
      pen += m;
    }
  }
  return base == ~0ull ? CHM_INF_COST : (int64_t)(base + a.K * pen);
}

__global__ void __launch_bounds__(BLOCK) k_expand32(ExpandArgs32 a) {
  // a lane owns two neighbouring plan indices per tile of 2 * BLOCK and stores them as one 16-byte word
  const uint32_t first = blockIdx.x * (EXPAND_PER * BLOCK) + 2 * threadIdx.x;
  int64_t cost[EXPAND_PER];
#pragma unroll
  for (int rep = 0; rep < EXPAND_PER; ++rep) {
    const uint32_t gid = first + (rep >> 1) * (2 * BLOCK) + (rep & 1);
    cost[rep] = expand_one(a, gid < a.count ? gid : a.count - 1);   // lanes past the end redo the last index
  }
  const bool aligned = (((uintptr_t)a.costs) & 15u) == 0;            // uniform
#pragma unroll
  for (int rep = 0; rep < EXPAND_PER; rep += 2) {
    const uint32_t gid = first + (rep >> 1) * (2 * BLOCK);
    // streamed out, never read back here
    if (aligned && gid + 1 < a.count) {
      typedef long long pair_t __attribute__((ext_vector_type(2)));
      pair_t v;
      v.x = cost[rep];
      v.y = cost[rep + 1];
      __builtin_nontemporal_store(v, (pair_t *)(a.costs + gid));
    } else {
      if (gid < a.count) __builtin_nontemporal_store(cost[rep], &a.costs[gid]);
      if (gid + 1 < a.count) __builtin_nontemporal_store(cost[rep + 1], &a.costs[gid + 1]);
    }
  }
}

// One stage lost nodes and its vector table is small: the table and the data of the partitions a workgroup's
// plan indices belong to (cost without penalty, peer stage times) are staged in LDS first, so that the vector
// memory path carries the stores and little else (with all three reads per plan index going through it the
// kernel was bound by the address and data path of the CU's texture unit at about 350 G plan indices/s).
constexpr int EXPAND_REC = 3;         // uint4 words per partition record: cost, 8 peer stage times

__global__ void __launch_bounds__(BLOCK) k_expand32_lds(ExpandArgs32 a, uint32_t max_parts) {
  extern __shared__ uint4 staged[];   // [R * stride / 4] rows, then [max_parts][EXPAND_REC] partition records
  const uint32_t R = a.R_joint.d;
  const uint32_t row_words = R * ((uint32_t)a.stride[0] / 4u);
  uint4 *rec = staged + row_words;
  const uint32_t tile_first = blockIdx.x * (EXPAND_PER * BLOCK);
  const uint32_t tile_last = min(tile_first + EXPAND_PER * BLOCK, a.count) - 1;   // tile_first < count by the grid size
  const uint32_t p_first = fast_div(a.first_rr + tile_first, a.R_joint);
  const uint32_t n_parts = min(fast_div(a.first_rr + tile_last, a.R_joint) - p_first + 1, max_parts);
  const uint4 *rows4 = (const uint4 *)a.rows[0];
  for (uint32_t i = threadIdx.x; i < row_words; i += BLOCK) staged[i] = rows4[i];
  for (uint32_t i = threadIdx.x; i < n_parts; i += BLOCK) {
    const uint32_t pl = a.first_part + p_first + i;
    const uint64_t b = a.base[pl];
    const uint4 *w4 = (const uint4 *)(a.weights + (size_t)pl * (DEV_MAX_AFF * 8));
    rec[i * EXPAND_REC] = make_uint4((uint32_t)b, (uint32_t)(b >> 32), 0u, 0u);
    rec[i * EXPAND_REC + 1] = w4[0];
    rec[i * EXPAND_REC + 2] = w4[1];
  }
  __syncthreads();
  const uint32_t first = tile_first + 2 * threadIdx.x;
  int64_t cost[EXPAND_PER];
#pragma unroll
  for (int rep = 0; rep < EXPAND_PER; ++rep) {
    uint32_t gid = first + (rep >> 1) * (2 * BLOCK) + (rep & 1);
    gid = gid < a.count ? gid : a.count - 1;                        // lanes past the end redo the last index
    const uint32_t idx = a.first_rr + gid;
    const uint32_t q = fast_div(idx, a.R_joint);
    const uint32_t rr = idx - q * R;
    uint32_t lp = q - p_first;
    lp = lp < n_parts ? lp : n_parts - 1;
    const uint4 head = rec[lp * EXPAND_REC], w_lo = rec[lp * EXPAND_REC + 1];
    const uint64_t base = (uint64_t)head.x | ((uint64_t)head.y << 32);
    uint32_t m;
    if (a.stride[0] == 4) {
      const uint4 row = staged[rr];
      m = max(max(__umul24(row.x, w_lo.x), __umul24(row.y, w_lo.y)), max(__umul24(row.z, w_lo.z), __umul24(row.w, w_lo.w)));
    } else {
      const uint4 w_hi = rec[lp * EXPAND_REC + 2];
      const uint4 row = staged[2 * rr], row2 = staged[2 * rr + 1];
      m = max(max(__umul24(row.x, w_lo.x), __umul24(row.y, w_lo.y)), max(__umul24(row.z, w_lo.z), __umul24(row.w, w_lo.w)));
      m = max(m, max(max(__umul24(row2.x, w_hi.x), __umul24(row2.y, w_hi.y)), max(__umul24(row2.z, w_hi.z), __umul24(row2.w, w_hi.w))));
    }
    cost[rep] = base == ~0ull ? CHM_INF_COST : (int64_t)(base + a.K * m);
  }
  const bool aligned = (((uintptr_t)a.costs) & 15u) == 0;            // uniform
#pragma unroll
  for (int rep = 0; rep < EXPAND_PER; rep += 2) {
    const uint32_t gid = first + (rep >> 1) * (2 * BLOCK);
    if (aligned && gid + 1 < a.count) {
      typedef long long pair_t __attribute__((ext_vector_type(2)));
      pair_t v;
      v.x = cost[rep];
      v.y = cost[rep + 1];
      __builtin_nontemporal_store(v, (pair_t *)(a.costs + gid));
    } else {
      if (gid < a.count) __builtin_nontemporal_store(cost[rep], &a.costs[gid]);
      if (gid + 1 < a.count) __builtin_nontemporal_store(cost[rep + 1], &a.costs[gid + 1]);
    }
  }
}

__global__ void k_fill_u32(uint32_t *p, uint32_t n, uint32_t v) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

template <typename Fn>
int by_peers(int p, Fn fn) {
  switch (p) {
    case 1: return fn(std::integral_constant<int, 1>());
    case 2: return fn(std::integral_constant<int, 2>());
    case 3: return fn(std::integral_constant<int, 3>());
    case 4: return fn(std::integral_constant<int, 4>());
    case 5: return fn(std::integral_constant<int, 5>());
    case 6: return fn(std::integral_constant<int, 6>());
    case 7: return fn(std::integral_constant<int, 7>());
    case 8: return fn(std::integral_constant<int, 8>());
    default: return 1;
  }
}

// queued: the variant that compacts the partitions that fit (and, in a bounded search, may still win) through a ring per wave
template <int STRAT>
int launch_by_stages(int sp, const FastLaunch &a, uint32_t blocks, uint32_t tile_bytes, hipStream_t st, bool queued = false) {
#define CHM_CASE(SPV)                                                                         \
  case SPV:                                                                                   \
    if (queued && (STRAT == 2 || a.s.incumbent != nullptr))                                   \
      hipLaunchKernelGGL((k_fast_search<SPV, STRAT, 2>), dim3(blocks), dim3(BLOCK), 0, st, a); \
    else if (queued)                                                                          \
      hipLaunchKernelGGL((k_fast_search<SPV, STRAT, (STRAT == 2 ? 2 : 1)>), dim3(blocks), dim3(BLOCK), 0, st, a); \
    else                                                                                      \
      hipLaunchKernelGGL((k_fast_search<SPV, STRAT>), dim3(blocks), dim3(BLOCK), tile_bytes, st, a); \
    return 0;
  switch (sp) {
#ifdef CHM_TUNING_SUBSET        // (-DCHM_TUNING_SUBSET: only the stage counts of the 32-card shape, for quick rebuilds while tuning)
    CHM_CASE(7) CHM_CASE(8)
#else
    CHM_CASE(2) CHM_CASE(3) CHM_CASE(4) CHM_CASE(5) CHM_CASE(6) CHM_CASE(7) CHM_CASE(8)
    CHM_CASE(9) CHM_CASE(10) CHM_CASE(11) CHM_CASE(12) CHM_CASE(13) CHM_CASE(14) CHM_CASE(15) CHM_CASE(16)
#endif
    default: return 1;
  }
#undef CHM_CASE
}

template <int STRAT>
int filter_by_stages(int sp, const ListFilter &a, uint32_t blocks, hipStream_t st) {
#define CHM_CASE(SPV)                                                                         \
  case SPV:                                                                                   \
    hipLaunchKernelGGL((k_list_filter<SPV, STRAT>), dim3(blocks), dim3(BLOCK), 0, st, a);      \
    return 0;
  switch (sp) {
#ifdef CHM_TUNING_SUBSET        // (-DCHM_TUNING_SUBSET: only the stage counts of the 32-card shape, for quick rebuilds while tuning)
    CHM_CASE(7) CHM_CASE(8)
#else
    CHM_CASE(2) CHM_CASE(3) CHM_CASE(4) CHM_CASE(5) CHM_CASE(6) CHM_CASE(7) CHM_CASE(8)
    CHM_CASE(9) CHM_CASE(10) CHM_CASE(11) CHM_CASE(12) CHM_CASE(13) CHM_CASE(14) CHM_CASE(15) CHM_CASE(16)
#endif
    default: return 1;
  }
#undef CHM_CASE
}

bool stages_covered(int sp) { return sp >= 2 && sp <= 16; }

// Share of uniformly drawn partitions into `sp` stages whose largest per-node peak memory stays within the cap
// (the filter of largest_peak, on the host).  Only steers the choice between two kernels with equal results.
constexpr int FIT_SAMPLES = 128;
constexpr float QUEUE_BELOW_SHARE = 0.80f;
float estimate_fit_share(const DevScenario &h, const FastFamily &ff, int strat, int sp) {
  const int L = h.L, k = sp - 1, n = L - 1;
  uint64_t state = 0x9e3779b97f4a7c15ull ^ ((uint64_t)L << 32) ^ ((uint64_t)sp << 8) ^ (uint64_t)strat;
  auto next = [&state]() {                   // splitmix64
    uint64_t z = (state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
  };
  int fit = 0;
  for (int smp = 0; smp < FIT_SAMPLES; ++smp) {
    // k distinct cut positions out of 1..n, each subset equally likely: for j = n-k+1..n draw t from 1..j and
    // take t, or j when t is already taken; the chosen positions are bits of a mask
    uint64_t chosen[2] = {0, 0};
    for (int j = n - k + 1; j <= n; ++j) {
      const int t = 1 + (int)(((next() >> 32) * (uint64_t)j) >> 32);
      const int pick = (chosen[t >> 6] >> (t & 63)) & 1 ? j : t;
      chosen[pick >> 6] |= 1ull << (pick & 63);
    }
    int c[DEV_MAX_S + 1];
    c[0] = 0;
    int filled = 1;
    for (int w = 0; w < 2; ++w)
      for (uint64_t m = chosen[w]; m; m &= m - 1) c[filled++] = w * 64 + __builtin_ctzll(m);
    c[sp] = L;
    int64_t st[DEV_MAX_S], ac[DEV_MAX_S];
    for (int s = 0; s < sp; ++s) { st[s] = h.pw[c[s + 1]] - h.pw[c[s]]; ac[s] = h.pa[c[s + 1]] - h.pa[c[s]]; }
    int64_t peak = 0;
    for (int s = 0; s < sp; ++s) {
      const int coef = ff.mem_coef[s];
      if (coef < 0) continue;
      const int64_t a = strat == 0 ? st[s] + st[(s + 1) % sp] : st[s];
      const int64_t b = strat == 0 ? ac[s] + ac[(s + 1) % sp] : ac[s];
      peak = std::max(peak, a + (ff.has_act ? b * coef : 0));
    }
    if (peak <= (int64_t)h.cap) ++fit;
  }
  return (float)fit / (float)FIT_SAMPLES;
}

}  // namespace

static void fast_quiesce(FastState *f) {
  if (f->quiesce) f->quiesce(f->owner);
}

// Run and vector tables of the rerouting family (see FastTables): enumeration on the host, rows decoded on the
// device, then the table block is uploaded again with the offsets and counts.  At load for families whose
// vectors are swept inside the search kernel, on first need for the large ones.  False on a failed HIP call;
// when table and count table disagree the strategy is handed back to the generic kernels (usable[2] = false).
// rows of the rank-ordered vector table, decoded on the device (queued on the library's stream, not waited for)
static bool build_vector_rows(FastState *f, const DevScenario &h) {
  const FastTables *t = &f->h_tables;
  hipStream_t ls = (hipStream_t)f->load_stream;
  if (!f->d_vecs && !pool_take(f->d_vecs, f->vec_words * sizeof(uint32_t))) return false;
  for (int a = 0; a < h.n_aff; ++a) {
    const int stride = h.aff_peers[a] <= 4 ? 4 : 8;
    hipLaunchKernelGGL(k_make_rows, dim3((t->vec_rows[a] + BLOCK - 1) / BLOCK), dim3(BLOCK), 0, ls, f->d_scn, f->d_comp, a,
                       f->d_vecs + t->vec_off[a], t->vec_rows[a], stride);
  }
  f->vecs_ready = hipGetLastError() == hipSuccess;
  return f->vecs_ready;
}

static bool build_reroute_tables(FastState *f, const DevScenario &h) {
  FastTables *t = &f->h_tables;
  // run tables (host enumeration in rank order: shared entries lexicographic, see FastTables)
  std::vector<uint32_t> runs;
  if (f->usable[2]) {
    // group tables for the sweep kernel of large reroute spaces (see k_sweep_groups)
    for (int a = 0; a < h.n_aff && f->split; ++a) {
      t->grp_cap[a] = 0;
      const int p = h.aff_peers[a], total = h.aff_total[a];
      const int cap = h.rcap > 0 ? std::min(h.rcap, total) : total;
      if (p < 3 || (cap != 8 && cap != 16)) continue;
      int same = -1;
      for (int b = 0; b < a; ++b)
        if (h.aff_peers[b] == p && h.aff_total[b] == total && t->grp_cap[b]) same = b;
      if (same >= 0) { t->grp_off[a] = t->grp_off[same]; t->grp_count[a] = t->grp_count[same]; t->grp_cap[a] = t->grp_cap[same]; continue; }
      const int q = p - 3;                                 // shared entries per group
      const size_t at = runs.size();
      uint64_t vectors = 0;
      uint32_t n_groups = 0;
      std::vector<int> pre(q + 1, 0);
      // odometer over the shared entries in lexicographic order (every entry 0..cap, what is left must fit the last three)
      int pos = 0, rem = total;
      bool fresh = true;
      for (;;) {
        if (pos == q) {
          const int lo = std::max(0, rem - 2 * cap), hi = std::min(cap, rem);
          if (lo <= hi) {
            uint32_t d[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int i = 0; i < q; ++i) d[i] = (uint32_t)pre[i];
            d[5] = (uint32_t)lo; d[6] = (uint32_t)(hi - lo + 1); d[7] = (uint32_t)rem;
            runs.insert(runs.end(), d, d + 8);
            for (int v = lo; v <= hi; ++v) {
              const int r2 = rem - v;
              vectors += (uint64_t)(std::min(cap, r2) - std::max(0, r2 - cap) + 1);
            }
            ++n_groups;
          }
          --pos;
          if (pos < 0) break;
          rem += pre[pos];
          ++pre[pos];
          fresh = false;
          continue;
        }
        if (fresh) pre[pos] = 0;
        if (pre[pos] > std::min(cap, rem)) {
          --pos;
          if (pos < 0) break;
          rem += pre[pos];
          ++pre[pos];
          fresh = false;
          continue;
        }
        rem -= pre[pos];
        ++pos;
        fresh = true;
      }
      if (vectors == h.aff_R[a] && n_groups > 0) {
        t->grp_off[a] = (uint32_t)at; t->grp_count[a] = n_groups; t->grp_cap[a] = (uint32_t)cap;
      } else {
        runs.resize(at);                                   // table and count disagree: the run sweep serves this stage
      }
    }
    // run tables of the stages that have no group table
    for (int a = 0; a < h.n_aff && f->usable[2]; ++a) {
      if (t->grp_cap[a] != 0) { t->run_off[a] = 0; t->run_count[a] = 0; continue; }
      int same = -1;
      for (int b = 0; b < a; ++b)
        if (h.aff_peers[b] == h.aff_peers[a] && h.aff_total[b] == h.aff_total[a]) same = b;
      if (same >= 0) {
        t->run_off[a] = t->run_off[same]; t->run_count[a] = t->run_count[same]; t->unrolled_shape[a] = t->unrolled_shape[same];
        continue;
      }
      const int p = h.aff_peers[a], total = h.aff_total[a];
      const int cap = h.rcap > 0 ? h.rcap : total;
      t->run_off[a] = (uint32_t)runs.size();
      uint64_t vectors = 0;
      uint32_t n_runs = 0;
      const int q = p >= 2 ? p - 2 : 0;                    // shared entries per run
      std::vector<int> pre(q + 1, 0);
      // odometer over the shared entries in lexicographic order
      int rem = total;
      int pos = 0;
      bool fresh = true;                                   // entering position `pos` from the left
      for (;;) {
        if (pos == q) {
          const int tail = p >= 2 ? 2 : 1;                 // entries left to fill
          const int lo = p >= 2 ? std::max(0, rem - cap) : rem, hi = p >= 2 ? std::min(cap, rem) : rem;
          if (lo <= hi && rem <= tail * cap) {
            uint32_t d[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int i = 0; i < q; ++i) d[i] = (uint32_t)pre[i];
            d[6] = (uint32_t)lo | ((uint32_t)rem << 16);
            d[7] = (uint32_t)(hi - lo + 1);
            runs.insert(runs.end(), d, d + 8);
            vectors += d[7];
            ++n_runs;
          }
          // step back to the previous position and advance it
          --pos;
          if (pos < 0) break;
          rem += pre[pos];
          ++pre[pos];
          fresh = false;
          continue;
        }
        if (fresh) pre[pos] = 0;
        if (pre[pos] > std::min(cap, rem)) {               // exhausted this position
          --pos;
          if (pos < 0) break;
          rem += pre[pos];
          ++pre[pos];
          fresh = false;
          continue;
        }
        rem -= pre[pos];
        ++pos;
        fresh = true;
      }
      t->run_count[a] = n_runs;
      if (vectors != h.aff_R[a]) f->usable[2] = false;     // table and count must agree
      if (h.rcap <= 0 || h.rcap >= total) {                // uncapped: every composition is valid
        const bool have = (p == 2 && (total == 8 || total == 16 || total == 32)) || (p == 3 && (total == 8 || total == 16));
        if (have) t->unrolled_shape[a] = (uint32_t)p * 256u + (uint32_t)total;
      }
    }
    if (!f->usable[2]) f->split = false;
  }
  if (!f->usable[2]) return true;
  if (runs.empty()) runs.assign(8, 0);
  fast_quiesce(f);                                           // (an earlier asynchronous call may still hold the placeholder)
  if (f->d_runs) pool_release(f->d_runs);
  if (f->d_vecs) pool_release(f->d_vecs);
  f->d_runs = nullptr; f->d_vecs = nullptr;
  // uploads and the row kernel run on the library's own stream and only that stream is waited for
  hipStream_t ls = (hipStream_t)f->load_stream;
  bool up = pool_take(f->d_runs, runs.size() * sizeof(uint32_t));
  up = up && pool_staged_upload(&f->stage, f->d_runs, runs.data(), runs.size() * sizeof(uint32_t), ls);
  up = up && pool_staged_upload(&f->stage, f->d_tables, t, sizeof(FastTables), ls);
  // the vector table itself (rank-ordered rows) only serves the cost store of plan indices; where the vectors are
  // swept by kernels of their own it is tens of MB and is built when a cost store first asks for it
  f->vecs_ready = false;
  if (up && !f->split) up = build_vector_rows(f, h);
  up = (hipStreamSynchronize(ls) == hipSuccess) && up;       // also when something failed: `runs` must outlive its copy
  f->stage.used = 0;
  f->reroute_tables_ready = up;
  return up;
}

// 0: the tables are there; 1: building them showed that the specialised kernels do not cover this family;
// negative: a HIP call failed
static int ensure_reroute_tables(FastState *f, const DevScenario &h) {
  if (f->reroute_tables_ready) return 0;
  if (!f->usable[2]) return 1;
  if (!build_reroute_tables(f, h)) return -1;
  return f->usable[2] && f->reroute_tables_ready ? 0 : 1;
}

void fast_select(FastState *f, const DevScenario &h, bool int32_ok) {
  for (bool &u : f->usable) u = false;
  f->split = false;
  f->mul24_reroute = false;
  f->vec_words = 16;
  memset(&f->h_tables, 0, sizeof(f->h_tables));
  if (!int32_ok) return;
  // memory side of the int32 kernels: doubled static sums plus the largest activation term stay below
  // 2^31, and the (doubled) activation sums fit the 24-bit multiply
  if (2 * h.pw[h.L] + 2 * h.pa[h.L] * (int64_t)DEV_MAX_S >= (1ll << 31) || 2 * h.pa[h.L] >= (1ll << 24)) return;
  // 24-bit multiplies in the reroute sweep need peer stage times below 2^24
  uint32_t q_aff = 65536;
  for (int a = 0; a < h.n_aff; ++a)
    for (int i = 0; i < h.aff_peers[a]; ++i) q_aff = std::max(q_aff, h.aff_q[a][i]);
  const bool w24 = (((h.pf[h.L] + h.pb[h.L]) * (int64_t)q_aff) >> 16) + 2 < (1ll << 24);
  f->mul24_reroute = w24;
  FastTables *t = &f->h_tables;
  size_t vec_words = 16;
  for (int k = 0; k < 3; ++k) {
    const DevFamily &fam = h.fam[k];
    if (!fam.n_part || !stages_covered(fam.stages)) continue;
    if (k == 1 && fam.fixed_step == CHM_INF_COST) continue;
    bool ok = true;
    FastFamily &ff = t->fam[k];
    ff.n_cls = fam.n_cls;
    ff.fixed_step = (int32_t)fam.fixed_step;
    ff.w_total = (int32_t)h.pw[h.L];
    for (int j = 0; j < DEV_MAX_S; ++j) ff.mem_coef[j] = fam.mem_coef[j];
    ff.has_act = h.pa[h.L] > 0 ? 1 : 0;
    ff.assign = h.assign;
    ff.allreduce = (int32_t)h.allreduce;
    ff.fixed_layers = (k == 1 && h.n_fixed > 0) ? h.p0_max_layers : 0;
    ff.node_exists = h.node_exists;
    // 24-bit multiplies in the sharper lower bound: micro-batches x (doubled) stage time, plus the prefix, below 2^31
    ff.lb_prefix = (2 * (h.pf[h.L] + h.pb[h.L]) < (1ll << 24)) && ((int64_t)(h.D * h.M + h.S) * 2 * (h.pf[h.L] + h.pb[h.L]) < (1ll << 31)) ? 1 : 0;
    if (k == 0 && h.allreduce > 0 && h.L > 64) continue;     // colour masks of the specialised kernel hold 64 colours
    for (int j = 0; j <= h.S; ++j) ff.w0[j] = (int32_t)h.pw[h.p0[j]];
    for (int ci = 0; ci < fam.n_cls && ok; ++ci) {
      const DevClass &c = fam.cls[ci];
      FastClass &fc = ff.cls[ci];
      fc.n = c.n; fc.M = c.M; fc.comm_total = (int32_t)((c.n - 1) * h.comm);
      fc.dead0 = fc.dead1 = 1 << 20;
      fc.unit = 1;
      fc.q_min = c.n > 0 ? c.q[0] : 65536u;
      for (int j = 0; j < c.n; ++j) {
        fc.q[j] = c.q[j];
        fc.q_min = std::min(fc.q_min, c.q[j]);
        if (c.q[j] != 65536u) fc.unit = 0;
        fc.wlo[j] = (int32_t)h.pw[h.p0[c.host[j]]];
        fc.whi[j] = (int32_t)h.pw[h.p0[c.host[j] + 1]];
      }
      // every one of the (M + stages) scaled stage times in the bound may round down by up to two
      fc.lb_slack = fc.unit ? 0 : 2 * (c.M + fam.stages);
      if (k == 0) {
        // which partition stages the chain skips (at most two, the kernel handles no more)
        int n_dead = 0, dead[DEV_MAX_S];
        for (int s = 0, j = 0; s < fam.stages; ++s) {
          if (j < c.n && c.src[j] == s) ++j;
          else dead[n_dead++] = s;
        }
        if (n_dead > 2 || c.n < 1) ok = false;
        if (n_dead >= 1) fc.dead0 = dead[0];
        if (n_dead >= 2) fc.dead1 = dead[1];
      } else if (c.n != fam.stages) {
        ok = false;
      }
    }
    if (k == 2 && ok) {
      uint64_t r_sum = 0;
      for (int a = 0; a < h.n_aff && ok; ++a) {
        if (h.aff_peers[a] > FAST_MAX_P || h.aff_R[a] > FAST_SPLIT_R || !w24) { ok = false; break; }
        const int stride = h.aff_peers[a] <= 4 ? 4 : 8;
        const uint32_t padded = (uint32_t)((h.aff_R[a] + 3) / 4 * 4);
        // stages with the same peer count, orphan count and cap share one table
        int same = -1;
        for (int b = 0; b < a; ++b)
          if (h.aff_peers[b] == h.aff_peers[a] && h.aff_total[b] == h.aff_total[a]) same = b;
        t->vec_rows[a] = padded;
        t->lb_mult[a] = (uint32_t)((h.aff_total[a] + h.aff_peers[a] - 1) / h.aff_peers[a]);
        t->lb_q[a] = h.aff_q[a][0];
        for (int i = 1; i < h.aff_peers[a]; ++i) t->lb_q[a] = std::min(t->lb_q[a], h.aff_q[a][i]);
        if (same >= 0) t->vec_off[a] = t->vec_off[same];
        else { t->vec_off[a] = (uint32_t)vec_words; vec_words += ((size_t)padded * stride + 15) / 16 * 16; }
        r_sum += h.aff_R[a];
      }
      f->split = ok && r_sum > FAST_FUSED_R;
    }
    f->usable[k] = ok;
    f->fit_share[k] = (ok && k != 2) ? -1.0f : 1.0f;      // sampled on first need
  }
  f->vec_words = vec_words;
}

int fast_prepare(FastState *f, const DevScenario &h, bool int32_ok, const DevScenario *d_scn, const uint64_t *d_comp) {
  fast_select(f, h, int32_ok);
  if (!f->usable[0] && !f->usable[1] && !f->usable[2]) return 0;
  FastTables *t = &f->h_tables;
  f->d_scn = d_scn;
  f->d_comp = d_comp;
  f->reroute_tables_ready = false;
  hipStream_t ls = (hipStream_t)f->load_stream;
  bool up = pool_take(f->d_tables, sizeof(FastTables));
  if (up && f->usable[2]) up = pool_take(f->d_rowkey, DEV_MAX_AFF * sizeof(uint64_t));
  if (up && f->usable[2] && !f->split) {
    // the vectors are swept inside the search kernel: the (small) tables are built now, behind one wait
    up = build_reroute_tables(f, h);
  } else {
    up = up && pool_take(f->d_runs, 8 * sizeof(uint32_t));          // placeholder until the tables are built (or for good)
    if (up) hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, ls, f->d_runs, 8u, 0u);
    up = up && pool_staged_upload(&f->stage, f->d_tables, t, sizeof(FastTables), ls);
    up = (hipStreamSynchronize(ls) == hipSuccess) && up;
    f->stage.used = 0;
  }
  return up ? 0 : 1;
}

namespace {

// scratch of the split rerouting path and of plan-index scoring: per partition of a pass the cost without
// penalties, the peer stage times and the best penalty per affected stage
bool ensure_scratch(FastState *f, uint64_t parts) {
  const uint32_t need = (uint32_t)std::min<uint64_t>(FAST_SUB, std::max<uint64_t>(parts, 1 << 12));
  if (f->d_base && f->d_weights && f->d_pen && f->d_fit_list && f->d_fit_count && f->scratch_parts >= need) return true;
  fast_quiesce(f);                                           // what is replaced may still be read by an asynchronous call
  if (f->d_fit_count) pool_release(f->d_fit_count);
  if (f->d_fit_list) pool_release(f->d_fit_list);
  if (f->d_pen) pool_release(f->d_pen);
  if (f->d_weights) pool_release(f->d_weights);
  if (f->d_base) pool_release(f->d_base);
  f->d_fit_count = nullptr; f->d_fit_list = nullptr; f->d_pen = nullptr; f->d_weights = nullptr; f->d_base = nullptr; f->scratch_parts = 0;
  bool ok = pool_take(f->d_base, (size_t)need * sizeof(uint64_t));
  ok = ok && pool_take(f->d_weights, (size_t)need * DEV_MAX_AFF * 8 * sizeof(uint32_t));
  ok = ok && pool_take(f->d_pen, (size_t)need * DEV_MAX_AFF * sizeof(uint32_t));
  ok = ok && pool_take(f->d_fit_list, (size_t)need * sizeof(uint32_t));
  ok = ok && pool_take(f->d_fit_count, 64);
  if (ok) f->scratch_parts = need;
  return ok;
}

// scratch of one pass over an explicit list of `entries` entries (at most LIST_SUB); grows when a longer pass comes
bool ensure_list_scratch(FastState *f, uint32_t entries) {
  uint32_t need = 1u << 16;
  while (need < entries) need <<= 1;
  if (f->d_cut_list && f->d_cut_pos && f->d_cut_count && f->list_capacity >= need) return true;
  fast_quiesce(f);                                           // what is replaced may still be read by an asynchronous call
  if (f->d_cut_count) pool_release(f->d_cut_count);
  if (f->d_cut_pos) pool_release(f->d_cut_pos);
  if (f->d_cut_list) pool_release(f->d_cut_list);
  f->d_cut_count = nullptr; f->d_cut_pos = nullptr; f->d_cut_list = nullptr; f->list_capacity = 0;
  bool ok = pool_take(f->d_cut_list, (size_t)need * sizeof(uint4));
  ok = ok && pool_take(f->d_cut_pos, (size_t)need * sizeof(uint32_t));
  ok = ok && pool_take(f->d_cut_count, (size_t)(need / (BLOCK * FILTER_TILES_BOUNDED) + 1) * sizeof(uint32_t));
  if (ok) f->list_capacity = need;
  return ok;
}

// Explicit list of partition ranks: per pass of LIST_SUB entries, filter + compaction, then the search kernel
// over the entries that fit.
int launch_list(FastState *f, const DevScenario &h, const SearchLaunch &a, hipStream_t st) {
  if (!ensure_list_scratch(f, std::min<uint32_t>(a.part_count, LIST_SUB))) return -1;
  const int sp = h.fam[a.strategy].stages;
  // a bounded search prunes the later passes against the best cost of the earlier ones: a short first pass
  // makes one known early
  const bool bounded = a.incumbent != nullptr && a.costs_out == nullptr;
  for (uint32_t done = 0; done < a.part_count;) {
    const uint32_t n = std::min<uint32_t>(bounded && done == 0 ? LIST_FIRST : LIST_SUB, a.part_count - done);
    const uint32_t tiles = bounded ? FILTER_TILES_BOUNDED : FILTER_TILES;
    const uint32_t blocks = (n + BLOCK * tiles - 1) / (BLOCK * tiles);   // one workgroup per region, both kernels
    ListFilter lf;
    lf.tiles = (int32_t)tiles;
    lf.incumbent = bounded ? a.incumbent : nullptr;
    lf.incumbent0 = a.incumbent0;
    lf.scn = a.scn; lf.tab = f->d_tables; lf.n = n; lf.pos_base = done;
    lf.ranks = a.ranks ? a.ranks + done : nullptr;
    lf.cuts = a.cuts ? a.cuts + (size_t)done * (size_t)(sp - 1) : nullptr;
    lf.costs_out = a.costs_out; lf.cut_list = (uint4 *)f->d_cut_list; lf.cut_pos = f->d_cut_pos; lf.cut_count = f->d_cut_count;
    int rc = a.strategy == 0 ? filter_by_stages<0>(sp, lf, blocks, st)
             : a.strategy == 1 ? filter_by_stages<1>(sp, lf, blocks, st) : filter_by_stages<2>(sp, lf, blocks, st);
    if (rc) return rc;
    FastLaunch fl;
    fl.s = a;
    fl.s.ranks = nullptr;
    fl.s.cuts = nullptr;
    fl.s.part_first = 0;
    fl.s.part_count = n;
    fl.tab = f->d_tables;
    fl.vecs = f->d_vecs;
    fl.runs = f->d_runs;
    fl.per_lane = tiles;                  // rounds per region
    fl.base_out = nullptr;
    fl.weights_out = nullptr;
    fl.cut_list = (const uint4 *)f->d_cut_list;
    fl.cut_pos = f->d_cut_pos;
    fl.cut_count = f->d_cut_count;
    rc = a.strategy == 0 ? launch_by_stages<0>(sp, fl, blocks, 0, st)
         : a.strategy == 1 ? launch_by_stages<1>(sp, fl, blocks, 0, st) : launch_by_stages<2>(sp, fl, blocks, 0, st);
    if (rc) return rc;
    if (hipGetLastError() != hipSuccess) return -1;
    done += n;
  }
  return 0;
}

int launch_search(FastState *f, const DevScenario &h, const SearchLaunch &a, uint64_t *base_out, uint32_t *weights_out,
                  hipStream_t st) {
  FastLaunch fl;
  fl.s = a;
  fl.cut_list = nullptr;
  fl.cut_pos = nullptr;
  fl.cut_count = nullptr;
  fl.tab = f->d_tables;
  fl.vecs = f->d_vecs;
  fl.runs = f->d_runs;
  fl.base_out = base_out;
  fl.weights_out = weights_out;
  // Run length per lane.  Runs of at most 32 partitions (longer ones leave too few workgroups to even out the
  // tail: 62.9 M partitions then make about 30 workgroups per compute unit, six rounds of the five that are
  // resident); spaces below 2^25 partitions get at least 16 workgroups per compute unit and correspondingly shorter
  // runs (measured on 10 to 15 M partitions: unranking once per 10 to 15 partitions costs less than the idle tail
  // of fewer, longer workgroups; runs of 5 to 7 were 1 to 8 % slower).  Small spaces: runs of 4 as long as that
  // still gives every resident wave slot (256 CUs x 5 workgroups x 256 lanes) a lane, then shorter.
  const uint64_t lanes_balanced = 256ull * 16 * BLOCK, lanes_resident = 256ull * 5 * BLOCK;
  uint64_t per = a.part_count / lanes_balanced;
  if (per < 4) per = std::min<uint64_t>(4, a.part_count / lanes_resident);
  per = std::max<uint64_t>(1, std::min<uint64_t>(per, 32));
  if (a.ranks != nullptr || a.jump_at != 0xffffffffu) per = 1;   // a list has no successor to walk to; a run must not straddle two windows
  else if (a.costs_out != nullptr) per = std::min<uint64_t>(per, 8);   // bounds the LDS tile of the cost store
  fl.per_lane = (uint32_t)per;
  const uint32_t tile_bytes = (a.costs_out != nullptr && per > 1) ? (uint32_t)(BLOCK * per * sizeof(int64_t)) : 0u;
  const uint64_t lanes = (a.part_count + per - 1) / per;
  const uint32_t blocks = (uint32_t)((lanes + BLOCK - 1) / BLOCK);
  const int sp = h.fam[a.strategy].stages;
  // pure range search of a family in which a good share of the partitions fails the memory filter
  // (a bounded search needs the ring: only there a wave decides what to evaluate before it evaluates)
  const bool pure_range = a.ranks == nullptr && a.costs_out == nullptr && base_out == nullptr;
  const bool queued = pure_range && (a.incumbent != nullptr ||
                                     (a.strategy != 2 && f->queue_mode != 0 &&
                                      (f->queue_mode > 0 || fast_fit_share(f, h, a.strategy) < QUEUE_BELOW_SHARE)));
  if (!queued) { fl.s.incumbent = nullptr; fl.s.evaluated = nullptr; }
  fl.capacity_penalty = (queued && a.strategy == 2 && f->split) ? 1 : 0;
  int rc;
  if (a.strategy == 0) rc = launch_by_stages<0>(sp, fl, blocks, tile_bytes, st, queued);
  else if (a.strategy == 1) rc = launch_by_stages<1>(sp, fl, blocks, tile_bytes, st, queued);
  else rc = launch_by_stages<2>(sp, fl, blocks, tile_bytes, st, queued);
  if (rc) return rc;
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace

namespace {
int64_t scale_floor_host(int64_t x, uint32_t q) {
  return q == 65536u ? x : std::max<int64_t>(0, ((x * (int64_t)q) >> 16) - 1);
}
}  // namespace

bool fast_candidates_build(const FastState *f, const DevScenario &h, int k, uint64_t incumbent, CandidateSet *out) {
  out->total = 0;
  if (k < 0 || k > 2 || !f->usable[k] || (k == 2 && f->split) || incumbent == ~0ull) return false;
  const FastTables &t = f->h_tables;
  const FastFamily &ff = t.fam[k];
  const int sp = h.fam[k].stages, L = h.L;
  if (sp < 2 || sp > 16 || L > 255) return false;
  const size_t W = (size_t)L + 1;
  out->stages = sp;
  out->L = L;
  out->ways.assign((size_t)sp * W * W, 0);
  out->low_pair.assign((size_t)sp * W, 0);
  if (incumbent < (uint64_t)h.reconf[k]) return true;                     // nothing can reach it
  const int64_t limit = (int64_t)((incumbent - (uint64_t)h.reconf[k]) / (uint64_t)h.K);   // largest step time that may still win
  if ((int64_t)ff.fixed_step > limit) return true;
  auto pc = [&](int x) { return h.pf[x] + h.pb[x]; };
  // stage s = layers [b, e) taken alone (strategies 1 and 2): lower bound of the step time it implies, and its memory
  auto single_ok = [&](int s, int b, int e) {
    if (k == 0) return true;
    const int coef = ff.mem_coef[s];
    if (coef >= 0 && (h.pw[e] - h.pw[b]) + (ff.has_act ? (h.pa[e] - h.pa[b]) * coef : 0) > h.cap) return false;
    const int64_t c = pc(e) - pc(b);
    int64_t lb = 0;
    for (int ci = 0; ci < ff.n_cls; ++ci) {
      const FastClass &cl = ff.cls[ci];
      int64_t v = (int64_t)cl.M * c + pc(b);
      // At nominal speed also the wait before the stage's first backward counts: that one cannot start before
      // micro-batch 0 has gone forward through every stage and backward through the stages behind this one,
      // by which time the stage has at most run its warm-up forwards and one more (stages - 1 - s + 1 of them)
      if (cl.unit && cl.M >= sp - s) v += std::max<int64_t>(0, (pc(L) - pc(e)) - (int64_t)(sp - 1 - s) * (h.pf[e] - h.pf[b]));
      lb = std::max(lb, std::max<int64_t>(0, scale_floor_host(v, cl.q_min) - cl.lb_slack) + cl.comm_total);
    }
    if (ff.allreduce > 0) lb += (int64_t)ff.allreduce * (e - b);
    if (k == 2)
      for (int a = 0; a < h.n_aff; ++a)
        if (h.aff_stage[a] == s) lb += (int64_t)t.lb_mult[a] * scale_floor_host(c, t.lb_q[a]);
    return lb <= limit;
  };
  // node s of the ring under redundant computation runs stages s and s+1 = layers [a, e)
  auto pair_ok = [&](int s, int a, int e) {
    const int coef = ff.mem_coef[s];
    if (coef >= 0 && (h.pw[e] - h.pw[a]) + (ff.has_act ? (h.pa[e] - h.pa[a]) * coef : 0) > h.cap) return false;
    const int64_t c = pc(e) - pc(a);
    for (int ci = 0; ci < ff.n_cls; ++ci) {
      const FastClass &cl = ff.cls[ci];
      if (s == cl.dead0 || s == cl.dead1) continue;
      if (std::max<int64_t>(0, scale_floor_host((int64_t)cl.M * c, cl.q_min) - cl.lb_slack) + cl.comm_total > limit) return false;
    }
    return true;
  };
  if (k == 0) {
    // both terms fall as the pair starts later: the allowed starts are those from the first one on from which all pass
    for (int s = 0; s + 1 < sp; ++s)
      for (int e = s + 2; e <= L; ++e) {
        int a = e - 2;
        while (a >= 0 && pair_ok(s, a, e)) --a;
        out->low_pair[(size_t)s * W + e] = (uint8_t)(a + 1);              // e - 1: no start passes
      }
  }
  auto ways = [&](int s, int a, int b) -> uint64_t & { return out->ways[((size_t)s * W + b) * W + a]; };
  for (int b = 1; b <= L - (sp - 1); ++b)
    if (single_ok(0, 0, b)) ways(0, 0, b) = 1;
  std::vector<uint64_t> from(W + 1);
  for (int s = 1; s < sp; ++s) {
    for (int a = s; a <= L - (sp - s); ++a) {
      // from[x] = ways to arrange stages 0..s-1 with stage s-1 = [x', a), x' >= x
      from[a] = 0;
      for (int x = a - 1; x >= 0; --x) from[x] = from[x + 1] + ways(s - 1, x, a);
      const int b_lo = a + 1, b_hi = s == sp - 1 ? L : L - (sp - 1 - s);
      for (int b = (s == sp - 1 ? L : b_lo); b <= b_hi; ++b) {
        if (!single_ok(s, a, b)) continue;
        const int lo = std::min<int>(std::max<int>(out->low_pair[(size_t)(s - 1) * W + b], s - 1), a);
        ways(s, a, b) = from[lo];
      }
    }
  }
  uint64_t total = 0;
  for (int a = sp - 1; a < L; ++a) total += ways(sp - 1, a, L);
  out->total = total;
  // what the enumeration reads: per (stage, end) the counts accumulated over the starts
  for (int s2 = 0; s2 < sp; ++s2)
    for (int b = 0; b <= L; ++b) {
      uint64_t *row = out->ways.data() + ((size_t)s2 * W + b) * W;
      for (int a = 1; a <= L; ++a) row[a] += row[a - 1];
    }
  static uint64_t next_serial = 0;
  out->serial = __atomic_add_fetch(&next_serial, 1, __ATOMIC_RELAXED);
  return true;
}

void fast_candidate_cuts(const CandidateSet &cs, uint64_t idx, uint8_t *cuts) {
  const size_t W = (size_t)cs.L + 1;
  int s = cs.stages - 1, end = cs.L;
  int start = candidate_start(cs.ways.data() + ((size_t)s * W + end) * W, s, end - 1, idx);
  for (;;) {
    cuts[s - 1] = (uint8_t)start;
    if (s == 1) break;
    const int first = std::max<int>(cs.low_pair[(size_t)(s - 1) * W + end], s - 1);
    const int below = first >= start - 1 ? start - 1 : candidate_start(cs.ways.data() + ((size_t)(s - 1) * W + start) * W, first, start - 1, idx);
    end = start;
    start = below;
    --s;
  }
}

int fast_candidates_search(FastState *f, const DevScenario &h, const SearchLaunch &a, const CandidateSet &cs, uint64_t stride,
                           void *stream) {
  if (cs.total == 0 || a.part_count == 0) return 0;
  if (a.part_count > CAND_PASS || a.idx_bits < 23 || stride < 1 || (a.part_first + a.part_count - 1) * stride >= cs.total) return 1;
  hipStream_t st = (hipStream_t)stream;
  const uint32_t total = a.part_count;
  const uint32_t blocks = (total + BLOCK - 1) / BLOCK;
  if (f->cand_capacity < total) {
    fast_quiesce(f);
    if (f->d_cand_list) pool_release(f->d_cand_list);
    if (f->d_cand_pos) pool_release(f->d_cand_pos);
    if (f->d_cand_count) pool_release(f->d_cand_count);
    f->d_cand_list = nullptr; f->d_cand_pos = nullptr; f->d_cand_count = nullptr; f->cand_capacity = 0;
    const uint64_t cap = std::max<uint64_t>(1 << 16, (uint64_t)blocks * BLOCK);
    bool ok = pool_take(f->d_cand_list, cap * sizeof(uint4));
    ok = ok && pool_take(f->d_cand_pos, cap * sizeof(uint32_t));
    ok = ok && pool_take(f->d_cand_count, cap / BLOCK * sizeof(uint32_t));
    if (!ok) return -1;
    f->cand_capacity = cap;
  }
  if (f->cand_ways_capacity < cs.ways.size()) {
    fast_quiesce(f);
    if (f->d_cand_ways) pool_release(f->d_cand_ways);
    if (f->d_cand_low) pool_release(f->d_cand_low);
    f->d_cand_ways = nullptr; f->d_cand_low = nullptr; f->cand_ways_capacity = 0; f->cand_serial = 0;
    bool ok = pool_take(f->d_cand_ways, cs.ways.size() * sizeof(uint64_t));
    ok = ok && pool_take(f->d_cand_low, cs.ways.size());      // more than stages x (L+1)
    if (!ok) return -1;
    f->cand_ways_capacity = cs.ways.size();
  }
  if (f->cand_serial != cs.serial) {
    // The tables go through a pinned staging buffer: a copy from pageable memory keeps the host busy until the data
    // has left (tens of microseconds for the 150 KB of the 32-card shape, during which nothing is launched), a copy
    // from pinned memory is queued and done.  An event tells when the buffer may be written again.
    f->cand_serial = 0;
    const size_t ways_bytes = cs.ways.size() * sizeof(uint64_t), low_bytes = cs.low_pair.size();
    if (f->cand_stage_capacity < ways_bytes + low_bytes) {
      if (f->cand_copied && hipEventSynchronize((hipEvent_t)f->cand_copied) != hipSuccess) return -1;
      if (f->h_cand_stage) pool_release(f->h_cand_stage);
      f->h_cand_stage = nullptr; f->cand_stage_capacity = 0;
      if (!pool_take_pinned(f->h_cand_stage, ways_bytes + low_bytes)) return -1;
      f->cand_stage_capacity = ways_bytes + low_bytes;
    }
    if (!f->cand_copied) {
      hipEvent_t ev = nullptr;
      if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) return -1;
      f->cand_copied = ev;
    } else if (hipEventSynchronize((hipEvent_t)f->cand_copied) != hipSuccess) {
      return -1;
    }
    memcpy(f->h_cand_stage, cs.ways.data(), ways_bytes);
    memcpy(f->h_cand_stage + ways_bytes, cs.low_pair.data(), low_bytes);
    if (hipMemcpyAsync(f->d_cand_ways, f->h_cand_stage, ways_bytes, hipMemcpyHostToDevice, st) != hipSuccess) return -1;
    if (hipMemcpyAsync(f->d_cand_low, f->h_cand_stage + ways_bytes, low_bytes, hipMemcpyHostToDevice, st) != hipSuccess) return -1;
    if (hipEventRecord((hipEvent_t)f->cand_copied, st) != hipSuccess) return -1;
    f->cand_serial = cs.serial;
  }
  CandidateEnum e;
  e.ways = f->d_cand_ways; e.low_pair = f->d_cand_low; e.stages = cs.stages; e.L = cs.L; e.total = total; e.first = a.part_first; e.stride = stride;
  e.cut_list = (uint4 *)f->d_cand_list; e.cut_pos = f->d_cand_pos; e.cut_count = f->d_cand_count;
  hipLaunchKernelGGL(k_enumerate_candidates, dim3(blocks), dim3(BLOCK), 0, st, e);
  FastLaunch fl;
  fl.s = a;
  fl.s.ranks = nullptr;
  fl.s.cuts = nullptr;
  fl.s.costs_out = nullptr;
  fl.s.part_first = 0;
  fl.s.part_count = total;
  fl.s.evaluated = nullptr;
  fl.tab = f->d_tables;
  fl.vecs = f->d_vecs;
  fl.runs = f->d_runs;
  fl.per_lane = 1;                        // one round per region of BLOCK candidates
  fl.base_out = nullptr;
  fl.weights_out = nullptr;
  fl.cut_list = (const uint4 *)f->d_cand_list;
  fl.cut_pos = f->d_cand_pos;
  fl.cut_count = f->d_cand_count;
  const int sp = h.fam[a.strategy].stages;
  const int rc = a.strategy == 0 ? launch_by_stages<0>(sp, fl, blocks, 0, st)
                 : a.strategy == 1 ? launch_by_stages<1>(sp, fl, blocks, 0, st) : launch_by_stages<2>(sp, fl, blocks, 0, st);
  if (rc) return rc;
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

float fast_fit_share(FastState *f, const DevScenario &h, int k) {
  if (k < 0 || k > 2) return 1.0f;
  if (f->fit_share[k] < 0.0f) f->fit_share[k] = estimate_fit_share(h, f->h_tables.fam[k], k, h.fam[k].stages);
  return f->fit_share[k];
}

bool fast_can_bound(const FastState *f, const SearchLaunch &a) {
  if (a.strategy < 0 || a.strategy > 2 || !f->usable[a.strategy]) return false;
  if (a.costs_out != nullptr) return false;
  if (a.ranks != nullptr || a.cuts != nullptr) return !(a.strategy == 2 && f->split);   // lists: bounded in their filter pass
  return true;                          // (large reroute spaces: least penalty from the peers' capacities)
}

int fast_search(FastState *f, const DevScenario &h, const SearchLaunch &a, void *stream) {
  if (a.strategy < 0 || a.strategy > 2 || !f->usable[a.strategy]) return 1;
  if (a.part_count == 0) return 0;
  hipStream_t st = (hipStream_t)stream;
  const bool list = a.ranks != nullptr || a.cuts != nullptr;
  if (!(a.strategy == 2 && f->split)) return list ? launch_list(f, h, a, st) : launch_search(f, h, a, nullptr, nullptr, st);
  // a bounded range search does without the sweep kernels: its queued kernel bounds and evaluates in one pass
  if (a.incumbent != nullptr && !list && a.costs_out == nullptr) return launch_search(f, h, a, nullptr, nullptr, st);
  if (list || a.costs_out != nullptr) return 1;   // the generic kernel handles lists for this shape
  if (const int rc = ensure_reroute_tables(f, h)) return rc;
  if (!ensure_scratch(f, a.part_count)) return -1;
  // split rerouting path, FAST_SUB partitions per pass: base costs and peer stage times, then one
  // sweep per affected stage over (partition blocks x row chunks), then the combine / argmin
  const FastTables &t = f->h_tables;
  for (uint32_t done = 0; done < a.part_count; done += FAST_SUB) {
    SearchLaunch sub = a;
    sub.part_first = a.part_first + done;
    sub.part_count = std::min<uint32_t>(FAST_SUB, a.part_count - done);
    int rc = launch_search(f, h, sub, f->d_base, f->d_weights, st);
    if (rc) return rc;
    const uint32_t n_pen = sub.part_count * DEV_MAX_AFF;
    hipLaunchKernelGGL(k_fill_u32, dim3((n_pen + 255) / 256), dim3(256), 0, st, f->d_pen, n_pen, 0xffffffffu);
    const uint32_t bx = (sub.part_count + BLOCK - 1) / BLOCK;
    for (int s = 0; s < h.n_aff && f->penalty_by_capacity; ++s) {
      const uint32_t total = (uint32_t)h.aff_total[s];
      hipLaunchKernelGGL(k_least_penalty, dim3(bx), dim3(BLOCK), 0, st, f->d_base, f->d_weights, f->d_pen, sub.part_count, s,
                         h.aff_peers[s], total, h.rcap > 0 ? (uint32_t)h.rcap : total);
    }
    bool compacted = false;
    for (int s = 0; s < h.n_aff && !f->penalty_by_capacity; ++s) {
      if (t.grp_cap[s] != 0) {
        // every lane a partition that fits: the list is built once per pass
        if (!compacted) {
          hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, f->d_fit_count, 1u, 0u);
          hipLaunchKernelGGL(k_compact_fit, dim3(bx), dim3(BLOCK), 0, st, f->d_base, sub.part_count, f->d_fit_list, f->d_fit_count);
          compacted = true;
        }
        const uint32_t n_groups = t.grp_count[s];
        // about 8192 workgroups in total, chunks of at least 128 groups (a lane works out its pair minima once per chunk)
        uint32_t chunks = std::max<uint32_t>(1, std::min<uint32_t>(8192 / bx + 1, n_groups / 128 + 1));
        chunks = std::min<uint32_t>(chunks, 65535);
        const uint32_t per_chunk = (n_groups + chunks - 1) / chunks;
        chunks = (n_groups + per_chunk - 1) / per_chunk;
        const uint32_t *groups = f->d_runs + t.grp_off[s];
        const bool cap16 = t.grp_cap[s] == 16;
        rc = by_peers(h.aff_peers[s], [&](auto tag) {
          constexpr int P = decltype(tag)::value;
          if constexpr (P >= 3) {
            if (cap16)
              hipLaunchKernelGGL((k_sweep_groups<P, 16>), dim3(bx, chunks), dim3(BLOCK), 0, st, groups, n_groups, per_chunk,
                                 f->d_fit_list, f->d_fit_count, f->d_weights, f->d_pen, s);
            else
              hipLaunchKernelGGL((k_sweep_groups<P, 8>), dim3(bx, chunks), dim3(BLOCK), 0, st, groups, n_groups, per_chunk,
                                 f->d_fit_list, f->d_fit_count, f->d_weights, f->d_pen, s);
            return 0;
          } else {
            return 1;
          }
        });
        if (rc) return -1;
        continue;
      }
      const uint32_t n_runs = t.run_count[s];
      // about 8192 workgroups in total, chunks of at least 64 runs
      uint32_t chunks = std::max<uint32_t>(1, std::min<uint32_t>(8192 / bx + 1, n_runs / 64 + 1));
      chunks = std::min<uint32_t>(chunks, 65535);
      const uint32_t per_chunk = (n_runs + chunks - 1) / chunks;
      chunks = (n_runs + per_chunk - 1) / per_chunk;
      const uint32_t *runs = f->d_runs + t.run_off[s];
      rc = by_peers(h.aff_peers[s], [&](auto tag) {
        constexpr int P = decltype(tag)::value;
        hipLaunchKernelGGL((k_sweep<P>), dim3(bx, chunks), dim3(BLOCK), 0, st, runs, n_runs, per_chunk, f->d_base,
                           f->d_weights, f->d_pen, sub.part_count, s);
        return 0;
      });
      if (rc) return -1;
    }
    hipLaunchKernelGGL(k_combine, dim3(bx), dim3(BLOCK), 0, st, f->d_base, f->d_pen, sub.part_count, h.n_aff,
                       (uint64_t)h.K, done, a.idx_bits, a.result);
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

int fast_score_reroute(FastState *f, const DevScenario &h, const DevScenario *d_scn, uint64_t local_first,
                       uint64_t count, int64_t *d_costs, void *stream) {
  if (!f->usable[2] || h.n_aff == 0) return 1;
  if (count == 0) return 0;
  if (const int rc = ensure_reroute_tables(f, h)) return rc;
  if (!f->vecs_ready) {
    if (!build_vector_rows(f, h) || hipStreamSynchronize((hipStream_t)f->load_stream) != hipSuccess) return -1;
  }
  hipStream_t st = (hipStream_t)stream;
  const FastTables &t = f->h_tables;
  const uint64_t R = h.fam[2].n_reroute;
  if (!ensure_scratch(f, (local_first + count - 1) / R - local_first / R + 1)) return -1;
  ExpandArgs e;
  memset(&e, 0, sizeof(e));
  e.base = f->d_base;
  e.weights = f->d_weights;
  e.n_aff = h.n_aff;
  for (int s = 0; s < h.n_aff; ++s) {
    e.rows[s] = f->d_vecs + t.vec_off[s];
    e.R[s] = h.aff_R[s];
    e.stride[s] = h.aff_peers[s] <= 4 ? 4 : 8;
    e.peers[s] = h.aff_peers[s];
  }
  e.R_joint = R;
  e.K = (uint64_t)h.K;
  const uint64_t last = local_first + count - 1;
  const uint64_t part_lo = local_first / R, part_hi = last / R;
  for (uint64_t p = part_lo; p <= part_hi; p += FAST_SUB) {
    const uint64_t np = std::min<uint64_t>(FAST_SUB, part_hi - p + 1);
    SearchLaunch sub = SearchLaunch();
    sub.scn = d_scn;
    sub.strategy = 2;
    sub.part_first = p;
    sub.part_count = (uint32_t)np;
    sub.idx_bits = 1;
    sub.result = f->d_rowkey;            // not written in this mode
    sub.feasible = f->d_rowkey + 1;      // scratch counter, not read
    int rc = launch_search(f, h, sub, f->d_base, f->d_weights, st);
    if (rc) return rc;
    // the plan indices of this pass: those of partitions [p, p+np) clipped to the request
    const uint64_t lo = std::max<uint64_t>(local_first, p * R);
    const uint64_t hi = std::min<uint64_t>(last, (p + np) * R - 1);
    e.local_first = lo;
    e.count = hi - lo + 1;
    e.part_base = p;
    e.costs = d_costs + (lo - local_first);
    if (R < (1ull << 31)) {
      // 32-bit index arithmetic: launches of at most 2^31 - 2^20 plan indices
      for (uint64_t done = 0; done < e.count;) {
        const uint64_t first = e.local_first + done;
        ExpandArgs32 x;
        memset(&x, 0, sizeof(x));
        x.base = e.base; x.weights = e.weights; x.n_aff = e.n_aff; x.K = e.K;
        for (int s = 0; s < h.n_aff; ++s) { x.rows[s] = e.rows[s]; x.R[s] = make_fast_div((uint32_t)e.R[s]); x.stride[s] = e.stride[s]; x.peers[s] = e.peers[s]; }
        x.R_joint = make_fast_div((uint32_t)R);
        x.first_part = (uint32_t)(first / R - p);
        x.first_rr = (uint32_t)(first % R);
        x.count = (uint32_t)std::min<uint64_t>(e.count - done, (1ull << 31) - (1ull << 20));
        x.costs = e.costs + done;
        // one affected stage with a table of at most 32 KB: rows and partition data through LDS
        const uint32_t row_bytes = (uint32_t)R * (uint32_t)x.stride[0] * 4u;
        const uint32_t max_parts = (uint32_t)((uint64_t)BLOCK * EXPAND_PER / R) + 2;
        if (h.n_aff == 1 && R >= 16 && row_bytes <= (32u << 10))
          hipLaunchKernelGGL(k_expand32_lds, dim3((x.count + BLOCK * EXPAND_PER - 1) / (BLOCK * EXPAND_PER)), dim3(BLOCK),
                             row_bytes + max_parts * EXPAND_REC * sizeof(uint4), st, x, max_parts);
        else
          hipLaunchKernelGGL(k_expand32, dim3((x.count + BLOCK * EXPAND_PER - 1) / (BLOCK * EXPAND_PER)), dim3(BLOCK), 0, st, x);
        done += x.count;
      }
      if (hipGetLastError() != hipSuccess) return -1;
      continue;
    }
    for (uint64_t done = 0; done < e.count;) {       // keep each grid below 2^31 blocks
      ExpandArgs part = e;
      part.local_first = e.local_first + done;
      part.count = std::min<uint64_t>(e.count - done, 1ull << 36);
      part.costs = e.costs + done;
      const uint32_t blocks = (uint32_t)((part.count + BLOCK - 1) / BLOCK);
      hipLaunchKernelGGL(k_expand, dim3(blocks), dim3(BLOCK), 0, st, part);
      done += part.count;
    }
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

void fast_release(FastState *f) {
  if (f->cand_copied) (void)hipEventDestroy((hipEvent_t)f->cand_copied);
  f->cand_copied = nullptr;
  if (f->h_cand_stage) pool_release(f->h_cand_stage);
  f->h_cand_stage = nullptr; f->cand_stage_capacity = 0;
  if (f->d_cand_low) pool_release(f->d_cand_low);
  if (f->d_cand_ways) pool_release(f->d_cand_ways);
  if (f->d_cand_count) pool_release(f->d_cand_count);
  if (f->d_cand_pos) pool_release(f->d_cand_pos);
  if (f->d_cand_list) pool_release(f->d_cand_list);
  f->d_cand_low = nullptr; f->d_cand_ways = nullptr; f->d_cand_count = nullptr; f->d_cand_pos = nullptr; f->d_cand_list = nullptr;
  f->cand_capacity = 0; f->cand_ways_capacity = 0;
  if (f->d_cut_count) pool_release(f->d_cut_count);
  if (f->d_cut_pos) pool_release(f->d_cut_pos);
  if (f->d_cut_list) pool_release(f->d_cut_list);
  f->d_cut_count = nullptr; f->d_cut_pos = nullptr; f->d_cut_list = nullptr; f->list_capacity = 0;
  if (f->d_rowkey) pool_release(f->d_rowkey);
  if (f->d_fit_count) pool_release(f->d_fit_count);
  if (f->d_fit_list) pool_release(f->d_fit_list);
  f->d_fit_count = nullptr; f->d_fit_list = nullptr;
  if (f->d_pen) pool_release(f->d_pen);
  if (f->d_weights) pool_release(f->d_weights);
  if (f->d_base) pool_release(f->d_base);
  if (f->d_vecs) pool_release(f->d_vecs);
  if (f->d_runs) pool_release(f->d_runs);
  if (f->d_tables) pool_release(f->d_tables);
  f->d_rowkey = nullptr; f->d_pen = nullptr; f->d_weights = nullptr; f->d_base = nullptr;
  f->d_vecs = nullptr;
  f->d_runs = nullptr;
  f->d_tables = nullptr;
}
