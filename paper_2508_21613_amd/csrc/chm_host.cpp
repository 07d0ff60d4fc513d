// Host side of libchm: the C-ABI of include/chm.h (and the measurement calls of include/chm_measure.h).  Validates a scenario, derives which
// recovery strategies exist for the failure set, lays out the plan index space and the
// device tables, and launches the scoring / search kernels.  No plan is ever scored on
// the host: without a working HIP device every compute entry point fails with CHM_ERR_HIP.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/chm.h"
#include "../../include/chm_measure.h"
#include "chm_dev.h"
#include "chm_fast.h"
#include "chm_internal.h"
#include "chm_pool.h"

// typed front ends of the caching allocator (chm_pool.h)
template <typename T>
static inline bool pool_take(T *&p, size_t bytes) { p = (T *)pool_device_alloc(bytes); return p != nullptr; }
template <typename T>
static inline bool pool_take_pinned(T *&p, size_t bytes) { p = (T *)pool_pinned_alloc(bytes); return p != nullptr; }

namespace {

typedef unsigned __int128 u128;

#define HIP_TRY(expr)                      \
  do {                                     \
    if ((expr) != hipSuccess) return CHM_ERR_HIP; \
  } while (0)

uint64_t add_sat(uint64_t a, uint64_t b) { return a > UINT64_MAX - b ? UINT64_MAX : a + b; }
uint64_t mul_sat(uint64_t a, uint64_t b) {
  u128 p = (u128)a * b;
  return p > (u128)UINT64_MAX ? UINT64_MAX : (uint64_t)p;
}
int bit_length(u128 v) { int n = 0; while (v) { ++n; v >>= 1; } return n; }

struct Slot { int strategy; uint64_t part_first; int idx_bits; uint32_t jump_at = 0xffffffffu; uint64_t jump_by = 0; };

}  // namespace

struct chm_scenario {
  chm_scenario();
  ~chm_scenario();
  chm_scenario(const chm_scenario &) = delete;
  chm_scenario &operator=(const chm_scenario &) = delete;
  DevScenario h;                         // host copy of what the device holds
  std::vector<uint64_t> comp;            // reroute count tables, all affected stages back to back
  std::vector<std::vector<int>> peers;   // per affected stage: surviving replicas, ascending
  std::vector<std::vector<uint8_t>> survivors;   // per pipeline: fault-free stage indices of its surviving nodes, ascending
  chm_space space;
  int device = 0;
  int smax = 4;                          // template bucket of the generic kernels
  int idx_bits = 0;                      // low bits of the packed argmin key
  bool int32_ok = false;                 // every intermediate of the recurrence fits in int32
  DevScenario *d_scn = nullptr;
  uint64_t *d_comp = nullptr;
  uint64_t *d_slots = nullptr;           // argmin words, one per launched chunk
  uint64_t *d_winner = nullptr;          // best reroute rank per affected stage
  uint64_t *d_xfer = nullptr;            // migration scheme: 8 bytes MiB to fetch + DEV_MAX_S bytes of stage indices
  uint64_t *d_result = nullptr;          // device-side address of h_pinned: k_finish_search writes its record straight there
  struct chm_search_state *search = nullptr;   // the search call in flight on this handle
  uint64_t *h_pinned = nullptr;          // pinned staging for the two small device-to-host copies
  uint32_t slot_words = 0;               // words d_slots has room for
  // d_slots as the last finished search left it: 0 = unknown (a fill kernel runs first); n > 0 = the words a search
  // of up to n chunks in the spread layout uses are in their initial state (filled once, and put back by
  // k_finish_search after every search since)
  uint32_t slots_ready_for = 0;
  bool timing = false;
  int bounded = 0;              // chm_set_bounded_search: 0 off, 1 on, 2 on with seeds and enumeration at any size
  hipEvent_t ev[8] = {};
  chm_timing last = {};
  // Work launched through the handle that no call has waited for yet (the asynchronous scoring calls, a call
  // that failed half way): per stream one event recorded behind it.  Waited for before the handle's buffers are
  // replaced or released, so that neither needs a device-wide wait.
  struct InFlight { hipStream_t stream; hipEvent_t event; bool busy; } in_flight[4] = {};
  bool in_flight_overflow = false;       // more streams than slots: fall back to waiting for the device
  hipEvent_t side_start = nullptr, side_done[4] = {};   // fork / join of the library's side streams (created on first use)
  FastState fast;                        // shape-specialised search path (chm_fast.hip)
};

namespace {

// Argmin words and feasibility counters of one search call live in one device buffer of SLOT_WORDS words.
// Each launched chunk and each of the three counters owns SLOT_WAYS words, SLOT_STRIDE words apart, when the
// call has few enough chunks for that; otherwise one word each.
enum { MAX_SLOTS = 1 << 16, SLOT_WORDS = (1 << 16) + 64, SLOT_WAYS = 16, SLOT_STRIDE = 16 };

// The library's own stream of a device (uploads, table kernels at load): created on first use, never destroyed,
// default priority, does not synchronise with the null stream.
hipStream_t load_stream_of(int device) {
  enum { MAX_DEVICES = 64 };
  static std::mutex lock;
  static hipStream_t streams[MAX_DEVICES] = {};
  if (device < 0 || device >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> hold(lock);
  if (!streams[device] && hipStreamCreateWithFlags(&streams[device], hipStreamNonBlocking) != hipSuccess) streams[device] = nullptr;
  return streams[device];
}

// records that work launched through the handle may still be running on `st`
void mark_in_flight(chm_scenario *s, hipStream_t st) {
  int slot = -1;
  for (int i = 0; i < 4; ++i)
    if (s->in_flight[i].busy && s->in_flight[i].stream == st) slot = i;
  for (int i = 0; i < 4 && slot < 0; ++i)
    if (!s->in_flight[i].busy) slot = i;
  if (slot < 0) { s->in_flight_overflow = true; return; }
  chm_scenario::InFlight &f = s->in_flight[slot];
  if (!f.event && hipEventCreateWithFlags(&f.event, hipEventDisableTiming) != hipSuccess) { f.event = nullptr; s->in_flight_overflow = true; return; }
  if (hipEventRecord(f.event, st) != hipSuccess) { s->in_flight_overflow = true; return; }
  f.stream = st;
  f.busy = true;
}

// waits until nothing launched through the handle is running any more (the handle's device must be current)
void quiesce(chm_scenario *s) {
  for (int i = 0; i < 4; ++i) {
    if (!s->in_flight[i].busy) continue;
    if (hipEventSynchronize(s->in_flight[i].event) != hipSuccess) s->in_flight_overflow = true;
    s->in_flight[i].busy = false;
  }
  if (s->in_flight_overflow) (void)hipDeviceSynchronize();
  s->in_flight_overflow = false;
}
void quiesce_owner(void *owner) { quiesce((chm_scenario *)owner); }

// Marks the stream of a call as possibly busy when the call ends, unless the call has waited for it itself.
struct StreamGuard {
  chm_scenario *s; hipStream_t st; bool armed = true;
  StreamGuard(chm_scenario *s_, void *stream) : s(s_), st((hipStream_t)stream) {}
  ~StreamGuard() { if (armed) mark_in_flight(s, st); }
  // rc of a call that ends with a wait for the stream on every path that returns one of these
  int settled(int rc) { if (rc == CHM_OK || rc == CHM_ERR_NO_FEASIBLE || rc == CHM_ERR_UNRECOVERABLE) armed = false; return rc; }
};

const chm_family *find_family(const chm_scenario *s, int strategy) {
  for (int i = 0; i < s->space.n_families; ++i)
    if (s->space.fam[i].strategy == strategy) return &s->space.fam[i];
  return nullptr;
}

bool same_class(const DevClass &a, const DevClass &b) {
  return a.n == b.n && a.M == b.M && !memcmp(a.src, b.src, sizeof(a.src)) && !memcmp(a.host, b.host, sizeof(a.host)) &&
         !memcmp(a.q, b.q, sizeof(a.q));
}

void add_class(DevClass *list, int32_t *n, const DevClass &c) {
  for (int i = 0; i < *n; ++i)
    if (same_class(list[i], c)) return;
  list[(*n)++] = c;
}

// micro-batches over pipelines in proportion to node counts, leftovers one by one from the
// first pipeline, empty pipelines refilled from the largest (Planner, "Batch Distribution")
void share_micro_batches(int D, int total, const int *nodes, int *out) {
  long long N = 0, given = 0;
  for (int d = 0; d < D; ++d) N += nodes[d];
  for (int d = 0; d < D; ++d) { out[d] = nodes[d] ? (int)((long long)total * nodes[d] / N) : 0; given += out[d]; }
  for (int d = 0, left = (int)(total - given); left > 0; d = (d + 1) % D)
    if (nodes[d]) { ++out[d]; --left; }
  for (;;) {
    int hole = -1, top = -1;
    for (int d = 0; d < D; ++d) {
      if (!nodes[d]) continue;
      if (out[d] == 0 && hole < 0) hole = d;
      if (top < 0 || out[d] > out[top]) top = d;
    }
    if (hole < 0 || top < 0 || out[top] < 2) return;
    --out[top]; ++out[hole];
  }
}

// number of vectors of `parts` entries in [0, cap] (cap<=0: unbounded) with a given sum,
// for every (parts' <= parts, sum' <= total): tab[parts' * (total+1) + sum']
void count_table(int parts, int total, int cap, std::vector<uint64_t> *tab) {
  const int stride = total + 1;
  tab->assign((size_t)(parts + 1) * stride, 0);
  (*tab)[0] = 1;
  for (int p = 1; p <= parts; ++p)
    for (int t = 0; t <= total; ++t) {
      uint64_t acc = 0;
      const int vmax = cap > 0 ? std::min(cap, t) : t;
      for (int v = 0; v <= vmax; ++v) acc = add_sat(acc, (*tab)[(size_t)(p - 1) * stride + (t - v)]);
      (*tab)[(size_t)p * stride + t] = acc;
    }
}

int validate(const chm_scenario_desc *d) {
  if (!d) return CHM_ERR_ARG;
  if (d->L < 1 || d->L > CHM_MAX_L || d->PP < 1 || d->PP > CHM_MAX_PP || d->PP > d->L || d->DP < 1 ||
      d->DP > CHM_MAX_DP || d->M < 1 || d->M > CHM_MAX_M || d->n_failed < 0 || d->n_failed > CHM_MAX_FAILED)
    return CHM_ERR_ARG;
  if (!d->fwd_us || !d->bwd_us || !d->mem_mib || (d->n_failed > 0 && !d->failed_nodes)) return CHM_ERR_ARG;
  if (d->comm_us < 0 || d->mem_cap_mib < 1 || d->horizon_steps < 1 || d->xfer_us_per_mib < 0) return CHM_ERR_ARG;
  if (d->transfer_assign < 0 || d->transfer_assign > 1 || d->allreduce_us < 0) return CHM_ERR_ARG;
  for (int i = 0; i < 3; ++i) if (d->reconf_us[i] < 0) return CHM_ERR_ARG;
  for (int l = 0; l < d->L; ++l)
    if (d->fwd_us[l] < 1 || d->bwd_us[l] < 1 || d->mem_mib[l] < 0 || (d->act_mib && d->act_mib[l] < 0)) return CHM_ERR_ARG;
  const int nodes = d->DP * d->PP;
  if (d->speed_q16)
    for (int n = 0; n < nodes; ++n)
      if (d->speed_q16[n] < 1 || d->speed_q16[n] > (1u << 20)) return CHM_ERR_ARG;
  for (int i = 0; i < d->n_failed; ++i) {
    if (d->failed_nodes[i] < 0 || d->failed_nodes[i] >= nodes) return CHM_ERR_ARG;
    for (int j = 0; j < i; ++j) if (d->failed_nodes[j] == d->failed_nodes[i]) return CHM_ERR_ARG;
  }
  return CHM_OK;
}

// Fills s->h, s->comp, s->peers and s->space from the description.
int build_model(const chm_scenario_desc *d, chm_scenario *s) {
  DevScenario &h = s->h;
  memset(&h, 0, sizeof(h));
  const int L = d->L, S = d->PP, D = d->DP, M = d->M;
  h.L = L; h.S = S; h.D = D; h.M = M;
  h.comm = d->comm_us; h.cap = d->mem_cap_mib; h.K = d->horizon_steps; h.xfer = d->xfer_us_per_mib;
  for (int i = 0; i < 3; ++i) h.reconf[i] = d->reconf_us[i];
  h.rcap = d->reroute_cap;
  h.assign = d->transfer_assign;
  h.allreduce = d->allreduce_us;
  for (int l = 0; l < L; ++l) {
    h.pf[l + 1] = h.pf[l] + d->fwd_us[l];
    h.pb[l + 1] = h.pb[l] + d->bwd_us[l];
    h.pw[l + 1] = h.pw[l] + d->mem_mib[l];
    h.pa[l + 1] = h.pa[l] + (d->act_mib ? d->act_mib[l] : 0);
  }
  for (int sgi = 0, pos = 0; sgi < S; ++sgi) {      // fault-free layout: extra layers on the last stages
    pos += L / S + (sgi >= S - L % S ? 1 : 0);
    h.p0[sgi + 1] = pos;
  }
  for (int i = 0; i < DEV_MAX_S; ++i)
    for (int x = 0; x < DEV_MAX_L; ++x) {
      uint64_t v;
      if (i == 0) v = 1;
      else if (x < i) v = 0;
      else if (x == i) v = 1;
      else v = add_sat(h.binom[i][x - 1], h.binom[i - 1][x - 1]);
      h.binom[i][x] = v;
    }

  bool dead[DEV_MAX_D][DEV_MAX_S] = {};
  uint32_t q[DEV_MAX_D][DEV_MAX_S];
  uint32_t qmax = 65536;
  for (int dd = 0; dd < D; ++dd)
    for (int j = 0; j < S; ++j) {
      q[dd][j] = d->speed_q16 ? d->speed_q16[dd * S + j] : 65536u;
      qmax = std::max(qmax, q[dd][j]);
    }
  int lost_in_pipe[DEV_MAX_D] = {}, lost_in_stage[DEV_MAX_S] = {};
  for (int i = 0; i < d->n_failed; ++i) {
    const int n = d->failed_nodes[i];
    dead[n / S][n % S] = true;
    ++lost_in_pipe[n / S];
    ++lost_in_stage[n % S];
  }

  for (int j = 0; j < S; ++j) {
    h.p0_max_layers = std::max(h.p0_max_layers, h.p0[j + 1] - h.p0[j]);
    for (int dd = 0; dd < D; ++dd)
      if (!dead[dd][j]) h.node_exists |= 1u << j;
  }
  s->survivors.assign(D, std::vector<uint8_t>());
  for (int dd = 0; dd < D; ++dd)
    for (int j = 0; j < S; ++j)
      if (!dead[dd][j]) s->survivors[dd].push_back((uint8_t)j);
  // ---- strategy 0: redundant computation; needs the ring predecessor of every failed node
  bool has0 = S >= 2;
  for (int dd = 0; dd < D; ++dd)
    for (int j = 0; j < S; ++j)
      if (dead[dd][j] && dead[dd][(j + S - 1) % S]) has0 = false;
  if (has0) {
    DevFamily &f = h.fam[0];
    f.strategy = 0; f.stages = S; f.doubled = 1;
    for (int dd = 0; dd < D; ++dd) {
      DevClass c; memset(&c, 0, sizeof(c));
      c.M = M;
      for (int j = 0; j < S; ++j)
        if (!dead[dd][j]) { c.src[c.n] = (uint8_t)j; c.host[c.n] = (uint8_t)j; c.q[c.n] = q[dd][j]; ++c.n; }
      add_class(f.cls, &f.n_cls, c);
    }
  }
  // ---- strategy 1: failed pipelines re-split over their survivors (all must keep the same count)
  int SB = 0;
  bool has1 = d->n_failed > 0;
  for (int dd = 0; dd < D; ++dd) {
    if (!lost_in_pipe[dd]) continue;
    const int left = S - lost_in_pipe[dd];
    if (left < 1 || (SB && left != SB)) has1 = false;
    SB = left;
  }
  if (has1) {
    DevFamily &f = h.fam[1];
    f.strategy = 1; f.stages = SB; f.doubled = 0;
    int nodes[DEV_MAX_D], mb[DEV_MAX_D];
    for (int dd = 0; dd < D; ++dd) nodes[dd] = S - lost_in_pipe[dd];
    share_micro_batches(D, D * M, nodes, mb);
    for (int dd = 0; dd < D; ++dd) {
      DevClass c; memset(&c, 0, sizeof(c));
      c.M = mb[dd];
      if (lost_in_pipe[dd]) {
        for (int j = 0; j < S; ++j)
          if (!dead[dd][j]) { c.src[c.n] = (uint8_t)c.n; c.host[c.n] = (uint8_t)j; c.q[c.n] = q[dd][j]; ++c.n; }
        add_class(f.cls, &f.n_cls, c);
      } else {
        for (int j = 0; j < S; ++j) { c.src[j] = (uint8_t)j; c.host[j] = (uint8_t)j; c.q[j] = q[dd][j]; }
        c.n = S;
        add_class(h.fixed, &h.n_fixed, c);
      }
    }
  }
  // ---- strategy 2: data rerouting; every stage must keep a peer and the capped split must exist
  bool has2 = true;
  uint64_t n_rr = 1;
  s->comp.clear(); s->peers.clear();
  for (int j = 0; j < S && has2; ++j) {
    if (!lost_in_stage[j]) continue;
    if (lost_in_stage[j] >= D) { has2 = false; break; }
    const int a = h.n_aff++;
    std::vector<int> pe;
    for (int dd = 0; dd < D; ++dd)
      if (!dead[dd][j]) { h.aff_q[a][pe.size()] = q[dd][j]; pe.push_back(dd); }
    s->peers.push_back(pe);
    h.aff_stage[a] = j; h.aff_peers[a] = (int)pe.size(); h.aff_total[a] = lost_in_stage[j] * M;
    std::vector<uint64_t> tab;
    count_table(h.aff_peers[a], h.aff_total[a], h.rcap, &tab);
    h.comp_off[a] = (uint32_t)s->comp.size();
    h.comp_stride[a] = (uint32_t)h.aff_total[a] + 1;
    h.aff_R[a] = tab[(size_t)h.aff_peers[a] * h.comp_stride[a] + h.aff_total[a]];
    s->comp.insert(s->comp.end(), tab.begin(), tab.end());
    if (h.aff_R[a] == 0) has2 = false;
    n_rr = mul_sat(n_rr, h.aff_R[a]);
  }
  if (!has2) { h.n_aff = 0; n_rr = 1; s->peers.clear(); }
  if (has2) {
    DevFamily &f = h.fam[2];
    f.strategy = 2; f.stages = S; f.doubled = 0;
    for (int dd = 0; dd < D; ++dd) {
      DevClass c; memset(&c, 0, sizeof(c));
      c.M = M; c.n = S;
      for (int j = 0; j < S; ++j) { c.src[j] = (uint8_t)j; c.host[j] = (uint8_t)j; c.q[j] = dead[dd][j] ? 65536u : q[dd][j]; }
      add_class(f.cls, &f.n_cls, c);
    }
  }
  if (s->comp.empty()) s->comp.push_back(1);
  // ---- per partition stage, the largest (pipeline length - position) among the nodes that run it
  for (int k = 0; k < 3; ++k) {
    DevFamily &f = h.fam[k];
    for (int j = 0; j < DEV_MAX_S; ++j) f.mem_coef[j] = -1;
    for (int ci = 0; ci < f.n_cls; ++ci)
      for (int j = 0; j < f.cls[ci].n; ++j)
        f.mem_coef[f.cls[ci].src[j]] = std::max<int32_t>(f.mem_coef[f.cls[ci].src[j]], f.cls[ci].n - j);
  }

  // ---- plan index space
  memset(&s->space, 0, sizeof(s->space));
  const bool has[3] = {has0, has1, has2};
  uint64_t off = 0;
  for (int k = 0; k < 3; ++k) {
    if (!has[k]) continue;
    DevFamily &f = h.fam[k];
    f.n_part = f.stages - 1 < DEV_MAX_S ? h.binom[f.stages - 1][L - 1] : UINT64_MAX;
    f.n_reroute = k == 2 ? n_rr : 1;
    const uint64_t total = mul_sat(f.n_part, f.n_reroute);
    if (f.n_part == UINT64_MAX || f.n_reroute == UINT64_MAX || total >= (1ull << 62) || add_sat(off, total) >= (1ull << 62))
      return CHM_ERR_OVERFLOW;
    chm_family &o = s->space.fam[s->space.n_families++];
    o.offset = off; o.n_part = f.n_part; o.n_reroute = f.n_reroute; o.stages = f.stages; o.strategy = k;
    off += total;
  }
  s->space.n_plans = off;

  // ---- bounds.  A pipeline time never exceeds (M + n - 1) x its largest stage time, a stage
  // time never exceeds twice the whole model (redundant computation) times the slowest factor.
  const u128 stage_max = (u128)(h.pf[L] + h.pb[L]) * 2 * ((qmax + 65535) / 65536);
  const u128 t_max = (u128)(D * M + S - 1) * stage_max + (u128)S * h.comm + (u128)L * h.allreduce;
  const u128 pen_max = (u128)CHM_MAX_FAILED * (CHM_MAX_FAILED * M) * stage_max;
  const u128 reconf_max = (u128)std::max(std::max(h.reconf[0], h.reconf[1]), h.reconf[2]) + (u128)h.xfer * h.pw[L];
  const u128 cost_max = (u128)h.K * (t_max + pen_max) + reconf_max;
  if (cost_max >= ((u128)1 << 62)) return CHM_ERR_OVERFLOW;
  // packed argmin key: cost in the high bits, chunk-local partition index in the low ones
  s->idx_bits = std::min(30, 64 - bit_length(cost_max + 1));
  if (s->idx_bits < 8) return CHM_ERR_OVERFLOW;
  // int32 recurrence is exact when even the largest intermediate (incl. the Q16 product's
  // result and the penalty) stays below 2^31
  s->int32_ok = (t_max + pen_max) < ((u128)1 << 31) && stage_max * 65536 < ((u128)1 << 62);
  const int widest = std::max(S, 1);
  s->smax = widest <= 4 ? 4 : widest <= 8 ? 8 : widest <= 16 ? 16 : 32;
  return CHM_OK;
}

void release(chm_scenario *s) {
  if (!s) return;
  // wait for what was launched through this handle and nothing else, then every buffer goes back to the allocator
  int current = 0;
  const bool switched = hipGetDevice(&current) == hipSuccess && current != s->device && hipSetDevice(s->device) == hipSuccess;
  quiesce(s);
  fast_release(&s->fast);
  for (auto &e : s->ev) if (e) (void)hipEventDestroy(e);
  for (auto &f : s->in_flight) if (f.event) (void)hipEventDestroy(f.event);
  if (s->side_start) (void)hipEventDestroy(s->side_start);
  for (auto &e : s->side_done) if (e) (void)hipEventDestroy(e);
  if (s->h_pinned) pool_release(s->h_pinned);
  if (s->d_xfer) pool_release(s->d_xfer);
  if (s->d_winner) pool_release(s->d_winner);
  if (s->d_slots) pool_release(s->d_slots);
  if (s->d_comp) pool_release(s->d_comp);
  if (s->d_scn) pool_release(s->d_scn);
  if (switched) (void)hipSetDevice(current);
  delete s;
}

void decode_partition(const chm_scenario *s, int k, uint64_t rank, uint8_t *cuts) {
  int x = s->h.L - 2;
  for (int i = k; i >= 1; --i) {
    while (s->h.binom[i][x] > rank) --x;
    cuts[i - 1] = (uint8_t)(x + 1);
    rank -= s->h.binom[i][x];
    --x;
  }
}

void decode_reroute(const chm_scenario *s, int a, uint64_t rank, uint16_t *row /* [16], by replica */) {
  const DevScenario &h = s->h;
  const uint64_t *tab = s->comp.data() + h.comp_off[a];
  int rem = h.aff_total[a];
  const int p = h.aff_peers[a];
  for (int pos = 0; pos < p; ++pos) {
    const int left = p - 1 - pos;
    int v = 0;
    for (;; ++v) {
      const uint64_t cnt = tab[(size_t)left * h.comp_stride[a] + (rem - v)];
      if (rank < cnt) break;
      rank -= cnt;
    }
    row[s->peers[a][pos]] = (uint16_t)v;
    rem -= v;
  }
}

void fill_plan(const chm_scenario *s, const chm_family *f, uint64_t part_rank, const uint64_t *rr_ranks, int64_t cost,
               chm_best *out) {
  memset(out, 0, sizeof(*out));
  uint64_t joint = 0;
  if (f->strategy == 2)
    for (int a = 0; a < s->h.n_aff; ++a) joint = joint * s->h.aff_R[a] + rr_ranks[a];
  out->index = f->offset + part_rank * f->n_reroute + joint;
  out->cost = cost;
  out->strategy = f->strategy;
  out->stages = f->stages;
  decode_partition(s, f->stages - 1, part_rank, out->cuts);
  if (f->strategy == 2) {
    out->n_affected = s->h.n_aff;
    for (int a = 0; a < s->h.n_aff; ++a) {
      out->affected_stage[a] = s->h.aff_stage[a];
      decode_reroute(s, a, rr_ranks[a], out->reroute[a]);
    }
  }
}

void nothing_found(chm_best *out) {
  memset(out, 0, sizeof(*out));
  out->index = UINT64_MAX;
  out->cost = CHM_INFEASIBLE;
}

// a range of partition ranks [first, first+count) of one strategy, or (ranks != null) a list of
// `count` partition ranks in device memory; costs (nullable, device) receives one cost per entry
// (cuts != null: the list holds rows of cut positions instead)
// (cand != null: a bounded search over the enumerated candidates of the whole family; count = their number,
// the key carries the candidate's index, `covers` = partitions of the family for the accounting)
struct Job {
  int strategy; uint64_t first, count; const uint64_t *ranks; int64_t *costs; const uint8_t *cuts = nullptr;
  const CandidateSet *cand = nullptr; uint64_t covers = 0; uint64_t stride = 1;
  bool seed = false;            // a few ranks searched ahead of their range for a good incumbent: left out of the accounting
  // two windows of ranks in one job (see SearchLaunch::jump_at): entries from jump_at on lie jump_by ranks further on;
  // only for jobs of a single chunk
  uint32_t jump_at = 0xffffffffu; uint64_t jump_by = 0;
};

// Rank of the partition into `stages` stages whose cuts follow the quantiles of a prefix table (forward +
// backward time, or memory): cut j at the first position where the prefix reaches j/stages of the total.
uint64_t balanced_rank(const chm_scenario *s, int stages, const int64_t *prefix_a, const int64_t *prefix_b) {
  const int L = s->h.L, k = stages - 1;
  const int64_t total = prefix_a[L] + (prefix_b ? prefix_b[L] : 0);
  uint64_t rank = 0;
  int prev = 0;
  for (int j = 1; j <= k; ++j) {
    int x = prev + 1;
    while (x < L - (stages - j) && (prefix_a[x] + (prefix_b ? prefix_b[x] : 0)) * stages < total * j) ++x;
    rank += s->h.binom[j][x - 1];
    prev = x;
  }
  return rank;
}

// below this many partitions the bounded range search costs no more than counting and enumerating candidates
constexpr uint64_t ENUMERATE_FROM = 1ull << 25;

uint64_t rank_of_cuts(const chm_scenario *s, int k, const uint8_t *cuts) {
  uint64_t rank = 0;
  for (int i = 1; i <= k; ++i) rank += s->h.binom[i][cuts[i - 1] - 1];
  return rank;
}

// The library's side streams (per device, created on first use, default priority, never destroyed).  The handles
// of a batched search are dealt out over them, so that the last workgroups of one handle's kernels run beside the
// first ones of the next handle's instead of leaving the device partly idle at every kernel boundary (the kernels
// of a failure sweep take 0.1 to 0.4 ms each; the three strategies of one large search gain nothing from it:
// measured).  The events that tie the side streams to the caller's stream belong to the batch's first handle.
enum { SIDE_STREAMS = 4, BATCH_MIN = 8 };
struct SideStreams { hipStream_t stream[SIDE_STREAMS]; bool ok; };
SideStreams *side_streams_of(int device) {
  enum { MAX_DEVICES = 64 };
  static std::mutex lock;
  static SideStreams all[MAX_DEVICES] = {};
  if (device < 0 || device >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> hold(lock);
  SideStreams &l = all[device];
  if (!l.ok) {
    bool ok = true;
    for (int k = 0; k < SIDE_STREAMS && ok; ++k) ok = hipStreamCreateWithFlags(&l.stream[k], hipStreamNonBlocking) == hipSuccess;
    l.ok = ok;
  }
  return l.ok ? &l : nullptr;
}

// fork: the side streams start behind what is in `st` now; join: `st` continues behind what is in them now
bool side_fork(chm_scenario *s, SideStreams *side, hipStream_t st) {
  bool ok = true;
  if (!s->side_start) {
    ok = hipEventCreateWithFlags(&s->side_start, hipEventDisableTiming) == hipSuccess;
    for (int k = 0; k < SIDE_STREAMS && ok; ++k) ok = hipEventCreateWithFlags(&s->side_done[k], hipEventDisableTiming) == hipSuccess;
  }
  ok = ok && hipEventRecord(s->side_start, st) == hipSuccess;
  for (int k = 0; k < SIDE_STREAMS && ok; ++k) ok = hipStreamWaitEvent(side->stream[k], s->side_start, 0) == hipSuccess;
  return ok;
}
bool side_join(chm_scenario *s, SideStreams *side, hipStream_t st) {
  bool ok = true;
  for (int k = 0; k < SIDE_STREAMS; ++k)
    ok = hipEventRecord(s->side_done[k], side->stream[k]) == hipSuccess && hipStreamWaitEvent(st, s->side_done[k], 0) == hipSuccess && ok;
  return ok;
}

// One search call in flight on a handle: what launch_jobs set up and collect_jobs needs.
struct SearchCtx {
  std::vector<Job> jobs;                 // (copies: a batch keeps them across the launches of other handles)
  std::vector<Slot> slots;
  std::vector<size_t> slot_job;          // index into jobs
  uint32_t ways = 1, stride = 1, chunk_words = 1, key_words = 0;
  bool bounded_used[3] = {false, false, false};
  int ev_of[3] = {-1, -1, -1};
  bool device_finish = false;            // the winner was picked by k_finish_search; one record waits in h_pinned
  bool light = false;
  bool empty = false;                    // nothing to search
};

}  // namespace

struct chm_search_state { SearchCtx ctx; };
chm_scenario::chm_scenario() : search(new (std::nothrow) chm_search_state()) {}
chm_scenario::~chm_scenario() { delete search; }

namespace {

// Launches the argmin over the given partition ranges on the stream (nothing is waited for).
// incumbent0: cost of a plan known before the call (a bounded search prunes against it), ~0 = none;
// bounded: range jobs skip partitions by their lower bound.
// light: only cost, strategy and partition of the winner are wanted (out->index = the partition's first plan
// index; reroute vectors and time terms are left out, which saves their kernels and a synchronisation).
// want_result: a winner will be collected (collect_jobs); otherwise the kernels only score into the jobs' buffers.
int launch_jobs(chm_scenario *s, const std::vector<Job> &jobs, bool want_result, hipStream_t st, uint64_t incumbent0, bool bounded,
                bool light) {
  HIP_TRY(hipSetDevice(s->device));
  s->last = chm_timing();
  SearchCtx &c = s->search->ctx;
  c = SearchCtx();
  c.jobs = jobs;
  c.light = light;
  const uint64_t chunk = 1ull << s->idx_bits;
  // spaces that need more chunks than there are argmin slots are refused before anything is sized by them
  uint64_t n_chunks = 0;
  for (const Job &j : jobs) n_chunks += j.count / chunk + 1;
  if (n_chunks > MAX_SLOTS) return CHM_ERR_OVERFLOW;
  for (size_t ji = 0; ji < jobs.size(); ++ji) {
    const Job &j = jobs[ji];
    for (uint64_t done = 0; done < j.count; done += chunk) {
      Slot slot{j.strategy, ((j.ranks || j.cuts) ? 0 : j.first) + done, s->idx_bits};
      slot.jump_at = j.jump_at; slot.jump_by = j.jump_by;
      c.slots.push_back(slot);
      c.slot_job.push_back(ji);
    }
  }
  if (c.slots.empty()) { c.empty = true; return CHM_OK; }
  if (c.slots.size() > MAX_SLOTS) return CHM_ERR_OVERFLOW;
  const bool spread = (c.slots.size() + 8) * SLOT_WAYS * SLOT_STRIDE <= s->slot_words;
  c.ways = spread ? SLOT_WAYS : 1; c.stride = spread ? SLOT_STRIDE : 1;
  if (c.slots.size() + 8 > s->slot_words) return CHM_ERR_LIMIT;    // (only the static buffer is that small)
  c.chunk_words = c.ways * c.stride;              // words one chunk (or one counter) owns
  c.key_words = (uint32_t)c.slots.size() * c.chunk_words;
  // Layout of d_slots: first three feasibility counters, three counters of evaluated partitions, what the seed jobs
  // count (not reported) and the incumbent cost of a bounded search, one chunk's worth of words each; behind these
  // eight the argmin words of the chunks.  (The fixed part in front lets a search find the buffer ready whatever
  // the number of chunks of the search before it was.)
  uint64_t *d_count = s->d_slots;
  uint64_t *d_evaluated = d_count + 3 * c.chunk_words;
  uint64_t *d_seed_count = d_count + 6 * c.chunk_words;
  uint64_t *d_incumbent = d_count + 7 * c.chunk_words;
  uint64_t *d_keys = s->d_slots + 8 * c.chunk_words;
  const uint32_t n_keys = (uint32_t)c.slots.size();
  const uint32_t ready_before = s->slots_ready_for;
  const bool ready = spread && n_keys <= ready_before;       // (a known cost travels in the launch arguments)
  s->slots_ready_for = 0;                          // until this call's own finish kernel is in the stream
  // (a fill in the spread layout covers at least the 16 chunks the finish kernel takes, so that later searches of
  // other strategy masks find their words ready as well)
  const uint32_t fill_keys = spread ? std::max<uint32_t>(n_keys, std::min<uint32_t>(FINISH_MAX_SLOTS, s->slot_words / c.chunk_words - 8)) : n_keys;
  if (!ready && chmk_init_search(s->d_slots, 7 * c.chunk_words, ~0ull, 8 * c.chunk_words, fill_keys * c.chunk_words, st)) return CHM_ERR_HIP;
  const uint32_t ready_after = ready ? ready_before : (spread ? fill_keys : 0);
  if (s->timing) HIP_TRY(hipEventRecord(s->ev[0], st));
  size_t si = 0;
  int ev_i = 1;
  bool plain = true;                         // range jobs only: the device can pick the winner
  // (one enumerated candidate set of a single pass is as good as a range: the finish kernel reads the winner's cuts
  // from the candidate list)
  int cand_jobs = 0, cand_slot = -1, cand_strategy = -1;
  {
    int slot_at = 0;
    for (const Job &j : jobs) {
      plain = plain && !j.ranks && !j.cuts;
      if (j.cand) {
        ++cand_jobs;
        cand_slot = slot_at; cand_strategy = j.strategy;
        plain = plain && j.stride == 1 && j.count <= chunk && j.count <= (uint64_t)CAND_PASS;
      }
      slot_at += (int)((j.count + chunk - 1) / chunk);
    }
    plain = plain && cand_jobs <= 1;
  }
  for (const Job &j : jobs) {
    for (uint64_t done = 0; done < j.count; done += chunk, ++si) {
      SearchLaunch a;
      a.scn = s->d_scn; a.comp = s->d_comp; a.strategy = j.strategy;
      a.part_first = j.first + done;
      a.part_count = (uint32_t)std::min<uint64_t>(chunk, j.count - done);
      a.jump_at = j.jump_at; a.jump_by = j.jump_by;
      a.incumbent0 = incumbent0;
      if (j.jump_at != 0xffffffffu && j.count > chunk) return CHM_ERR_ARG;        // (two-window jobs are a few dozen ranks)
      a.idx_bits = s->idx_bits;
      a.result = d_keys + si * c.chunk_words;
      a.feasible = j.seed ? d_seed_count : d_count + (size_t)j.strategy * c.chunk_words;
      a.slot_mask = c.ways - 1;
      a.slot_stride = c.stride;
      a.ranks = j.ranks ? j.ranks + done : nullptr;
      a.cuts = j.cuts ? j.cuts + (size_t)done * (size_t)(s->h.fam[j.strategy].stages - 1) : nullptr;
      a.costs_out = j.costs ? j.costs + done : nullptr;
      if (j.cand) {
        a.incumbent = d_incumbent;
        if (fast_candidates_search(&s->fast, s->h, a, *j.cand, j.stride, st)) return CHM_ERR_HIP;
        continue;
      }
      if (bounded && fast_can_bound(&s->fast, a)) {
        a.incumbent = d_incumbent;
        a.evaluated = j.seed ? d_seed_count : d_evaluated + (size_t)j.strategy * c.chunk_words;
        c.bounded_used[j.strategy] = !(j.ranks || j.cuts);   // lists: what passes their filter is evaluated and counted as fitting
      }
      int rc = fast_search(&s->fast, s->h, a, st);      // > 0: shape not covered by a specialised kernel
      if (rc > 0) rc = chmk_search(a, s->smax, st);
      if (rc) return CHM_ERR_HIP;
    }
    if (j.seed) continue;
    const uint64_t covered = j.cand ? j.covers : j.count;
    s->last.partitions[j.strategy] += covered;
    uint64_t per_part = 1;
    if (j.strategy == 2 && s->h.n_aff) { per_part = 0; for (int a = 0; a < s->h.n_aff; ++a) per_part += s->h.aff_R[a]; }
    s->last.evaluations[j.strategy] += covered * per_part;
    if (s->timing && ev_i < 7) { HIP_TRY(hipEventRecord(s->ev[ev_i], st)); c.ev_of[j.strategy] = ev_i; ++ev_i; }
  }
  if (!want_result) return CHM_OK;
  // Few chunks of plain ranges: a one-workgroup kernel behind the search kernels picks the winner, adds up the
  // counters and computes the winner's transition time (and its best reroute vectors), so the host waits once
  // and reads one record.
  if (plain && c.slots.size() <= FINISH_MAX_SLOTS && c.ways <= FINISH_MAX_WAYS) {
    FinishArgs f;
    memset(&f, 0, sizeof(f));
    f.scn = s->d_scn; f.slots = d_keys; f.counters = d_count;
    f.n_slots = (uint32_t)c.slots.size(); f.ways = c.ways; f.stride = c.stride; f.idx_bits = s->idx_bits;
    f.sweep_winner = light ? 0 : ((s->fast.split && s->fast.usable[2]) ? 2 : 1);
    f.comp = s->d_comp;
    for (size_t i = 0; i < FINISH_MAX_SLOTS; ++i) f.jump_at[i] = 0xffffffffu;
    f.cand_slot = cand_jobs == 1 ? cand_slot : -1;
    f.cand_k = cand_jobs == 1 ? s->h.fam[cand_strategy].stages - 1 : 0;
    f.cand_cuts = cand_jobs == 1 ? s->fast.d_cand_list : nullptr;
    for (size_t i = 0; i < c.slots.size(); ++i) {
      f.strategy[i] = c.slots[i].strategy; f.part_first[i] = c.slots[i].part_first;
      f.jump_at[i] = c.slots[i].jump_at; f.jump_by[i] = c.slots[i].jump_by;
    }
    f.out = s->d_result;                       // pinned host memory: no copy behind the kernel
    f.reset = spread ? 1 : 0;
    if (chmk_finish_search(f, s->smax, st)) return CHM_ERR_HIP;
    if (spread) s->slots_ready_for = ready_after;
    c.device_finish = true;
    return CHM_OK;
  }
  HIP_TRY(hipMemcpyAsync(s->h_pinned, s->d_slots, (size_t)(8 * c.chunk_words + c.key_words) * sizeof(uint64_t), hipMemcpyDeviceToHost, st));
  return CHM_OK;
}

// per-strategy kernel times of the call from the events launch_jobs recorded (the stream has been waited for)
int read_timing(chm_scenario *s) {
  const SearchCtx &c = s->search->ctx;
  if (!s->timing) return CHM_OK;
  int prev = 0;
  for (int k = 0; k < 3; ++k) {
    if (c.ev_of[k] < 0) continue;
    float ms = 0;
    // families are launched in strategy order, so each one's span starts at the previous event
    HIP_TRY(hipEventElapsedTime(&ms, s->ev[prev], s->ev[c.ev_of[k]]));
    s->last.family_ms[k] += ms;
    prev = c.ev_of[k];
  }
  HIP_TRY(hipEventElapsedTime(&s->last.total_ms, s->ev[0], s->ev[prev]));
  return CHM_OK;
}

// Second half of a search whose launch_jobs(want_result) succeeded: waits for the stream (unless the caller
// has: synced), reads the winner and fills *out.
int collect_jobs(chm_scenario *s, chm_best *out, uint64_t *position, hipStream_t st, bool synced) {
  SearchCtx &c = s->search->ctx;
  if (c.empty) { nothing_found(out); return CHM_ERR_NO_FEASIBLE; }
  HIP_TRY(hipSetDevice(s->device));
  if (!synced && hipStreamSynchronize(st) != hipSuccess) { s->slots_ready_for = 0; return CHM_ERR_HIP; }
  const bool light = c.light;
  int64_t best_cost = CHM_INFEASIBLE;
  int best_strategy = -1;
  uint64_t best_part = 0;
  uint64_t rr[DEV_MAX_AFF] = {};
  if (c.device_finish) {
    const uint64_t *rec = s->h_pinned;
    for (int k = 0; k < 3; ++k) { s->last.feasible[k] += rec[FINISH_COUNTS + k]; s->last.evaluated[k] += rec[FINISH_COUNTS + 3 + k]; }
    for (int k = 0; k < 3; ++k)
      if (!c.bounded_used[k]) s->last.evaluated[k] = s->last.feasible[k];
    if (const int rc = read_timing(s)) return rc;
    if (rec[FINISH_STRATEGY] == ~0ull) { nothing_found(out); return CHM_ERR_NO_FEASIBLE; }
    best_cost = (int64_t)rec[FINISH_COST];
    best_strategy = (int)rec[FINISH_STRATEGY];
    best_part = rec[FINISH_PART];
    if (light) {
      fill_plan(s, find_family(s, best_strategy), best_part, rr, best_cost, out);
      return CHM_OK;
    }
    if (best_strategy == 2)
      for (int a = 0; a < s->h.n_aff; ++a) rr[a] = rec[FINISH_RR + a];
    fill_plan(s, find_family(s, best_strategy), best_part, rr, best_cost, out);
    const int64_t t_trans = (int64_t)rec[FINISH_TRANS];
    if (t_trans < 0 || t_trans > best_cost || (best_cost - t_trans) % s->h.K != 0) return CHM_ERR_HIP;   // cannot happen
    out->t_trans_us = t_trans;
    out->t_step_us = (best_cost - t_trans) / s->h.K;
    return CHM_OK;
  }
  const uint32_t ways = c.ways, stride = c.stride, chunk_words = c.chunk_words;
  for (int k = 0; k < 3; ++k)
    for (uint32_t w = 0; w < ways; ++w) {
      s->last.feasible[k] += s->h_pinned[(size_t)k * chunk_words + (size_t)w * stride];
      s->last.evaluated[k] += s->h_pinned[(size_t)(3 + k) * chunk_words + (size_t)w * stride];
    }
  // kernels that evaluate everything that fits do not count what they evaluate
  for (int k = 0; k < 3; ++k)
    if (!c.bounded_used[k]) s->last.evaluated[k] = s->last.feasible[k];
  if (const int rc = read_timing(s)) return rc;
  // lowest cost; among equal costs the lowest plan index (strategy, then partition)
  const Job *best_job = nullptr;
  for (size_t i = 0; i < c.slots.size(); ++i) {
    uint64_t key = CHM_KEY_NONE;
    for (uint32_t w = 0; w < ways; ++w) key = std::min(key, s->h_pinned[(8 + i) * (size_t)chunk_words + (size_t)w * stride]);
    if (key == CHM_KEY_NONE) continue;
    const Job &job = c.jobs[c.slot_job[i]];
    const int64_t cost = (int64_t)(key >> c.slots[i].idx_bits);
    const uint64_t local = key & ((1ull << c.slots[i].idx_bits) - 1);
    uint64_t part = c.slots[i].part_first + local + (local >= c.slots[i].jump_at ? c.slots[i].jump_by : 0);
    if (job.cand) {                                // a candidate's index: its partition rank decides among equal costs
      uint8_t cuts[32];
      fast_candidate_cuts(*job.cand, part * job.stride, cuts);
      part = rank_of_cuts(s, s->h.fam[c.slots[i].strategy].stages - 1, cuts);
    }
    if (cost < best_cost || (cost == best_cost && (c.slots[i].strategy < best_strategy ||
                                                   (c.slots[i].strategy == best_strategy && part < best_part)))) {
      best_cost = cost;
      best_strategy = c.slots[i].strategy;
      best_part = part;
      best_job = &job;
    }
  }
  if (best_strategy < 0) { nothing_found(out); return CHM_ERR_NO_FEASIBLE; }
  if (best_job->ranks || best_job->cuts) {
    // list job: best_part is a position in the caller's list; fetch (or compute, on the device) the
    // partition rank behind it
    if (position) *position = best_part;
    const uint64_t *d_rank = best_job->ranks ? best_job->ranks + best_part : s->d_xfer;
    if (best_job->cuts) {
      const int k = s->h.fam[best_strategy].stages - 1;
      if (chmk_rank_cuts(s->d_scn, k, best_job->cuts + (size_t)best_part * (size_t)k, 1, s->d_xfer, st)) return CHM_ERR_HIP;
    }
    HIP_TRY(hipMemcpyAsync(s->h_pinned, d_rank, sizeof(uint64_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    best_part = s->h_pinned[0];
  }
  if (light) {
    fill_plan(s, find_family(s, best_strategy), best_part, rr, best_cost, out);
    return CHM_OK;
  }
  // the winner's reroute vectors (rerouting only) and its transition time, from the device, behind one
  // synchronisation; its step time follows from cost = horizon x step + transition
  const bool rerouted = best_strategy == 2 && s->h.n_aff > 0;
  if (rerouted) {
    const int32_t by_capacity = (s->fast.split && s->fast.usable[2]) ? 1 : 0;     // too many vectors for a one-lane sweep
    if (chmk_reroute_winner(s->d_scn, s->d_comp, best_part, by_capacity, s->d_winner, s->smax, st)) return CHM_ERR_HIP;
    HIP_TRY(hipMemcpyAsync(s->h_pinned, s->d_winner, DEV_MAX_AFF * sizeof(uint64_t), hipMemcpyDeviceToHost, st));
  }
  if (chmk_plan_transition(s->d_scn, best_strategy, best_part, (int64_t *)s->d_xfer, s->smax, st)) return CHM_ERR_HIP;
  HIP_TRY(hipMemcpyAsync(s->h_pinned + DEV_MAX_AFF, s->d_xfer, sizeof(int64_t), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  if (rerouted)
    for (int a = 0; a < s->h.n_aff; ++a) rr[a] = s->h_pinned[a];
  fill_plan(s, find_family(s, best_strategy), best_part, rr, best_cost, out);
  const int64_t t_trans = (int64_t)s->h_pinned[DEV_MAX_AFF];
  if (t_trans < 0 || t_trans > best_cost || (best_cost - t_trans) % s->h.K != 0) return CHM_ERR_HIP;   // cannot happen
  out->t_trans_us = t_trans;
  out->t_step_us = (best_cost - t_trans) / s->h.K;
  return CHM_OK;
}

// Runs the argmin over the given partition ranges.
// With out == null the kernels are only launched (asynchronous scoring into the jobs' cost buffers).
int run_jobs(chm_scenario *s, const std::vector<Job> &jobs, chm_best *out, uint64_t *position, hipStream_t st,
             uint64_t incumbent0, bool bounded, bool light = false) {
  const int rc = launch_jobs(s, jobs, out != nullptr, st, incumbent0, bounded, light);
  if (rc || !out) return rc;
  return collect_jobs(s, out, position, st, false);
}

// Exhaustive search, or (chm_set_bounded_search) the same argmin with the plans skipped that cannot reach it.
// A bounded search first evaluates a few partitions that are likely to be good: 64 ranks around the
// time-balanced and around the memory-balanced partition of every range.  Their best cost bounds everything
// else.  A family that is searched as a whole is then reduced on the host to its candidates, the partitions
// whose lower bound of the cost does not exceed that cost (see CandidateSet), and only those are enumerated and
// evaluated; sub-ranges, families with too many candidates and the shapes the candidate path does not cover are
// searched range by range with the bound applied per run and per partition.  The seeds' best plan competes
// with the result (it is among the candidates as well; equal plans compare equal).
// seeds of a bounded search: 64 ranks around the time-balanced and the memory-balanced partition of every range
std::vector<Job> make_seeds(const chm_scenario *s, const std::vector<Job> &given) {
  const uint64_t seeds_from = s->bounded == 2 ? 1 : (1u << 16);
  std::vector<Job> seeds;
  for (const Job &j : given) {
    if (j.ranks || j.cuts || j.costs || j.count < seeds_from) continue;
    const int stages = s->h.fam[j.strategy].stages;
    if (stages < 2) continue;
    const uint64_t at[2] = {balanced_rank(s, stages, s->h.pf, s->h.pb), balanced_rank(s, stages, s->h.pw, nullptr)};
    // the windows around the two ranks, in ascending order; one launch covers both (one job of two windows, or a
    // single window where they touch or one is empty)
    uint64_t lo[2], hi[2];
    for (int i = 0; i < 2; ++i) {
      const uint64_t mid = i == 0 ? std::min(at[0], at[1]) : std::max(at[0], at[1]);
      lo[i] = std::max<uint64_t>(j.first, mid >= 32 ? mid - 32 : 0);
      hi[i] = std::max(lo[i], std::min<uint64_t>(j.first + j.count, mid + 32));
    }
    if (lo[1] <= hi[0]) { hi[0] = std::max(hi[0], hi[1]); lo[1] = hi[1] = hi[0]; }      // overlapping or adjacent: one window
    if (hi[0] == lo[0]) { lo[0] = lo[1]; hi[0] = hi[1]; lo[1] = hi[1] = hi[0]; }          // first one empty
    if (lo[0] < hi[0]) {
      Job seed{j.strategy, lo[0], (hi[0] - lo[0]) + (hi[1] - lo[1]), nullptr, nullptr};
      seed.seed = true;
      if (lo[1] < hi[1]) { seed.jump_at = (uint32_t)(hi[0] - lo[0]); seed.jump_by = lo[1] - hi[0]; }
      seeds.push_back(seed);
    }
  }
  return seeds;
}

// Families that are enumerated need the seeds' cost on the host first.  When none can be (sub-ranges, families
// small enough that the range search costs no more), the seeds simply run ahead of the ranges in one pass.
bool any_enumerable(const chm_scenario *s, const std::vector<Job> &given) {
  const uint64_t enumerate_from = s->bounded == 2 ? 1 : ENUMERATE_FROM;
  bool any = false;
  for (const Job &j : given)
    any = any || (!j.ranks && !j.cuts && !j.costs && j.first == 0 && j.count == s->h.fam[j.strategy].n_part &&
                  j.count >= enumerate_from && s->idx_bits >= 23);
  return any;
}

int run_search(chm_scenario *s, const std::vector<Job> &given, chm_best *out, uint64_t *position, hipStream_t st) {
  s->fast.penalty_by_capacity = s->bounded && out != nullptr;
  if (!(s->bounded && out != nullptr)) return run_jobs(s, given, out, position, st, ~0ull, false);
  const uint64_t enumerate_from = s->bounded == 2 ? 1 : ENUMERATE_FROM;
  const std::vector<Job> seeds = make_seeds(s, given);
  if (!any_enumerable(s, given)) {
    std::vector<Job> all(seeds);
    all.insert(all.end(), given.begin(), given.end());
    return run_jobs(s, all, out, position, st, ~0ull, true);
  }
  chm_best seed_best;
  int seed_rc = CHM_ERR_NO_FEASIBLE;
  if (!seeds.empty()) {
    seed_rc = run_jobs(s, seeds, &seed_best, nullptr, st, ~0ull, false, true);
    if (seed_rc != CHM_OK && seed_rc != CHM_ERR_NO_FEASIBLE) return seed_rc;
  }
  uint64_t incumbent = seed_rc == CHM_OK ? (uint64_t)seed_best.cost : ~0ull;
  std::vector<CandidateSet> sets(given.size());
  std::vector<Job> jobs;
  uint64_t skipped[3] = {0, 0, 0};                     // partitions of families the bound excludes as a whole
  for (size_t i = 0; i < given.size(); ++i) {
    const Job &j = given[i];
    const bool whole = !j.ranks && !j.cuts && !j.costs && j.first == 0 && j.count == s->h.fam[j.strategy].n_part;
    bool listed = false;
    if (whole && incumbent != ~0ull && s->idx_bits >= 23) {
      // A family within reach of a range search is enumerated only when its candidates are few; one beyond it,
      // whenever they can be made few enough: while there are too many, a sample of them spread evenly over
      // their index order is evaluated, which lowers the incumbent and with it the number of candidates.
      // (below 2^25 partitions the range search costs no more than counting and enumerating does)
      const bool in_reach = j.count <= (1ull << 27);
      for (int round = 0; round < 8 && j.count >= enumerate_from; ++round) {
        if (!fast_candidates_build(&s->fast, s->h, j.strategy, incumbent, &sets[i])) break;
        const uint64_t total = sets[i].total;
        if (total <= (in_reach ? (uint64_t)CAND_DIRECT : (uint64_t)CAND_MAX)) { listed = true; break; }
        if (in_reach) break;
        Job sample{j.strategy, 0, CAND_SAMPLE, nullptr, nullptr};
        sample.cand = &sets[i];
        sample.stride = total / CAND_SAMPLE;
        chm_best found;
        const int rc_s = run_jobs(s, std::vector<Job>{sample}, &found, nullptr, st, incumbent, false, true);
        if (rc_s != CHM_OK && rc_s != CHM_ERR_NO_FEASIBLE) return rc_s;
        if (rc_s != CHM_OK || (uint64_t)found.cost >= incumbent) break;          // the sample found nothing better
        incumbent = (uint64_t)found.cost;
        seed_best = found;
        seed_rc = CHM_OK;
      }
    }
    if (listed) {
      if (sets[i].total == 0) { skipped[j.strategy] += j.count; continue; }
      for (uint64_t first = 0; first < sets[i].total; first += CAND_PASS) {
        Job c{j.strategy, first, std::min<uint64_t>(CAND_PASS, sets[i].total - first), nullptr, nullptr};
        c.cand = &sets[i];
        c.covers = first == 0 ? j.count : 0;
        jobs.push_back(c);
      }
    } else {
      jobs.push_back(j);
    }
  }
  int rc = run_jobs(s, jobs, out, position, st, incumbent, true);
  if (rc != CHM_OK && rc != CHM_ERR_NO_FEASIBLE) return rc;
  for (int k = 0; k < 3; ++k) {
    s->last.partitions[k] += skipped[k];
    uint64_t per_part = 1;
    if (k == 2 && s->h.n_aff) { per_part = 0; for (int a = 0; a < s->h.n_aff; ++a) per_part += s->h.aff_R[a]; }
    s->last.evaluations[k] += skipped[k] * per_part;
  }
  // The plan the incumbent came from lies inside the ranges just searched and passes every bound against its
  // own cost, so it has been found again unless something better was.  Should it ever be missing, it is
  // evaluated once more for its full description.
  if (seed_rc == CHM_OK && (rc == CHM_ERR_NO_FEASIBLE || seed_best.cost < out->cost)) {
    const chm_family *f = find_family(s, seed_best.strategy);
    const uint64_t part = (seed_best.index - f->offset) / f->n_reroute;
    return run_jobs(s, std::vector<Job>{Job{seed_best.strategy, part, 1, nullptr, nullptr}}, out, position, st, ~0ull, false);
  }
  return rc;
}


// Allocates the device side of a scenario whose host model is complete and uploads its tables.
// Takes ownership of s: on failure it is released and *out stays null.
int upload_scenario(chm_scenario *s, chm_scenario **out) {
  bool ok = hipGetDevice(&s->device) == hipSuccess;
  // everything the load puts on the device goes through the library's own stream, and only that stream is waited
  // for: searches other threads have in flight on their streams are not disturbed
  hipStream_t ls = ok ? load_stream_of(s->device) : nullptr;
  ok = ok && ls != nullptr;
  s->fast.load_stream = ls;
  s->fast.quiesce = quiesce_owner;
  s->fast.owner = s;
  ok = ok && pool_take(s->d_scn, sizeof(DevScenario));
  ok = ok && pool_take(s->d_comp, s->comp.size() * sizeof(uint64_t));
  ok = ok && pool_take(s->d_slots, (size_t)SLOT_WORDS * sizeof(uint64_t));
  s->slot_words = SLOT_WORDS;
  ok = ok && pool_take(s->d_winner, DEV_MAX_AFF * sizeof(uint64_t));
  ok = ok && pool_take(s->d_xfer, sizeof(uint64_t) + DEV_MAX_S);
  ok = ok && pool_take_pinned(s->h_pinned, (size_t)SLOT_WORDS * sizeof(uint64_t));
  ok = ok && hipHostGetDevicePointer((void **)&s->d_result, s->h_pinned, 0) == hipSuccess && s->d_result != nullptr;
  // uploads go through the handle's pinned buffer (nothing else uses it before the first search); the first 64
  // bytes stay free for the word the device sends back below
  if (ok) { s->fast.stage.base = (unsigned char *)s->h_pinned; s->fast.stage.bytes = (size_t)SLOT_WORDS * sizeof(uint64_t); s->fast.stage.used = 64; }
  ok = ok && pool_staged_upload(&s->fast.stage, s->d_scn, &s->h, sizeof(DevScenario), ls);
  ok = ok && pool_staged_upload(&s->fast.stage, s->d_comp, s->comp.data(), s->comp.size() * sizeof(uint64_t), ls);
  for (auto &e : s->ev) ok = ok && hipEventCreate(&e) == hipSuccess;
  const bool fixed = ok && s->h.fam[1].n_part;
  if (fixed) {
    // the healthy pipelines' step time under the fault-free layout is computed by the device
    ok = chmk_fixed_pipelines(s->d_scn, s->smax, ls) == 0;
    ok = ok && hipMemcpyAsync(s->h_pinned, &s->d_scn->fam[1].fixed_step, sizeof(int64_t), hipMemcpyDeviceToHost, ls) == hipSuccess;
  }
  if (ls) ok = (hipStreamSynchronize(ls) == hipSuccess) && ok;
  s->fast.stage.used = 0;
  if (ok && fixed) s->h.fam[1].fixed_step = (int64_t)s->h_pinned[0];
  ok = ok && fast_prepare(&s->fast, s->h, s->int32_ok, s->d_scn, s->d_comp) == 0;
  if (!ok) { release(s); return CHM_ERR_HIP; }
  *out = s;
  return CHM_OK;
}

}  // namespace

extern "C" int chm_load_scenario(const chm_scenario_desc *desc, chm_scenario **out) {
  if (!out) return CHM_ERR_ARG;
  *out = nullptr;
  int rc = validate(desc);
  if (rc) return rc;
  chm_scenario *s = new (std::nothrow) chm_scenario();
  if (!s || !s->search) { delete s; return CHM_ERR_HIP; }
  rc = build_model(desc, s);
  if (rc) { delete s; return rc; }
  return upload_scenario(s, out);
}

void chm_internal_share_micro_batches(int D, int total, const int *nodes, int *out) { share_micro_batches(D, total, nodes, out); }

// A scenario that holds one stand-alone pipeline of n stages and M micro-batches on identical
// nodes: its only family is the re-partition one (a single pipeline class, no untouched
// pipelines), with horizon 1 and no transition terms, so a plan's cost is the pipeline's 1F1B
// time plus comm per stage boundary and chm_search_best returns the best split of the layers.
int chm_internal_load_pipeline(int32_t L, const int32_t *fwd_us, const int32_t *bwd_us, const int32_t *mem_mib,
                               const int32_t *act_mib, int32_t n, int32_t M, int32_t comm_us, int32_t mem_cap_mib,
                               chm_scenario **out) {
  *out = nullptr;
  chm_scenario_desc d;
  memset(&d, 0, sizeof(d));
  d.L = L; d.PP = n; d.DP = 1; d.M = M;
  d.fwd_us = fwd_us; d.bwd_us = bwd_us; d.mem_mib = mem_mib; d.act_mib = act_mib;
  d.comm_us = comm_us; d.mem_cap_mib = mem_cap_mib; d.horizon_steps = 1;
  int rc = validate(&d);
  if (rc) return rc;
  chm_scenario *s = new (std::nothrow) chm_scenario();
  if (!s || !s->search) { delete s; return CHM_ERR_HIP; }
  rc = build_model(&d, s);          // no failure: strategies 0 and 2 of the intact pipeline; replaced below
  if (rc) { delete s; return rc; }
  DevScenario &h = s->h;
  for (int k = 0; k < 3; ++k) { DevFamily &f = h.fam[k]; memset(&f, 0, sizeof(f)); for (int j = 0; j < DEV_MAX_S; ++j) f.mem_coef[j] = -1; }
  h.n_aff = 0; h.n_fixed = 0;
  DevFamily &f = h.fam[1];
  f.strategy = 1; f.stages = n; f.doubled = 0; f.n_cls = 1; f.n_reroute = 1;
  f.n_part = h.binom[n - 1][L - 1];
  DevClass &c = f.cls[0];
  c.n = n; c.M = M;
  for (int j = 0; j < n; ++j) { c.src[j] = (uint8_t)j; c.host[j] = (uint8_t)j; c.q[j] = 65536u; f.mem_coef[j] = n - j; }
  memset(&s->space, 0, sizeof(s->space));
  if (f.n_part == UINT64_MAX || f.n_part >= (1ull << 62)) { delete s; return CHM_ERR_OVERFLOW; }
  s->space.n_families = 1;
  s->space.fam[0].offset = 0; s->space.fam[0].n_part = f.n_part; s->space.fam[0].n_reroute = 1;
  s->space.fam[0].stages = n; s->space.fam[0].strategy = 1;
  s->space.n_plans = f.n_part;
  return upload_scenario(s, out);
}

extern "C" int chm_kernel_selection(const chm_scenario_desc *desc, chm_selection *out) {
  if (!out) return CHM_ERR_ARG;
  memset(out, 0, sizeof(*out));
  int rc = validate(desc);
  if (rc) return rc;
  chm_scenario *s = new (std::nothrow) chm_scenario();
  if (!s || !s->search) { delete s; return CHM_ERR_HIP; }
  rc = build_model(desc, s);
  if (rc == CHM_OK) {
    fast_select(&s->fast, s->h, s->int32_ok);
    out->idx_bits = s->idx_bits;
    out->int32_recurrence = s->int32_ok ? 1 : 0;
    for (int k = 0; k < 3; ++k) {
      out->present[k] = s->h.fam[k].n_part ? 1 : 0;
      out->specialised[k] = s->fast.usable[k] ? 1 : 0;
      out->sharp_bound[k] = s->fast.usable[k] ? s->fast.h_tables.fam[k].lb_prefix : 0;
    }
    out->reroute_mul24 = s->fast.mul24_reroute ? 1 : 0;
    out->reroute_swept_apart = s->fast.split ? 1 : 0;
  }
  delete s;
  return rc;
}

extern "C" int chm_plan_space(const chm_scenario *s, chm_space *out) {
  if (!s || !out) return CHM_ERR_ARG;
  *out = s->space;
  return CHM_OK;
}

extern "C" int chm_score_plans(chm_scenario *s, uint64_t first, uint64_t count, int64_t *d_costs, void *hip_stream) {
  if (!s || (count && !d_costs)) return CHM_ERR_ARG;
  if (first > s->space.n_plans || count > s->space.n_plans - first) return CHM_ERR_RANGE;
  HIP_TRY(hipSetDevice(s->device));
  StreamGuard guard(s, hip_stream);                  // asynchronous: the stream stays marked as busy
  uint64_t lo = first, hi = first + count;
  for (int i = 0; i < s->space.n_families; ++i) {
    const chm_family &f = s->space.fam[i];
    const uint64_t fb = f.offset, fe = f.offset + f.n_part * f.n_reroute;
    const uint64_t a = std::max(lo, fb), b = std::min(hi, fe);
    if (a >= b) continue;
    if (f.n_reroute == 1) {
      // one plan per partition: the search kernels score the range and store every cost
      std::vector<Job> jobs;
      jobs.push_back({f.strategy, a - fb, b - a, nullptr, d_costs + (a - first)});
      const int rc = run_search(s, jobs, nullptr, nullptr, (hipStream_t)hip_stream);
      if (rc) return rc;
      continue;
    }
    {
      const int rc = f.strategy == 2 ? fast_score_reroute(&s->fast, s->h, s->d_scn, a - fb, b - a, d_costs + (a - first), hip_stream) : 1;
      if (rc < 0) return CHM_ERR_HIP;
      if (rc == 0) continue;             // > 0: shape not covered, the generic kernel below scores it
    }
    // split very long ranges so that the grid stays within 2^31 blocks
    for (uint64_t p = a; p < b;) {
      const uint64_t n = std::min<uint64_t>(b - p, 1ull << 36);
      if (chmk_score(s->d_scn, s->d_comp, f.strategy, p - fb, n, d_costs + (p - first), s->smax, hip_stream)) return CHM_ERR_HIP;
      p += n;
    }
  }
  return CHM_OK;
}

extern "C" int chm_score_ranks(chm_scenario *s, int32_t strategy, const uint64_t *d_part_ranks, uint64_t n,
                               int64_t *d_costs, void *hip_stream) {
  if (!s || strategy < 0 || strategy > 2 || (n && (!d_part_ranks || !d_costs))) return CHM_ERR_ARG;
  const chm_family *f = find_family(s, strategy);
  if (!f) return CHM_ERR_UNRECOVERABLE;
  if (f->n_reroute != 1) return CHM_ERR_ARG;
  HIP_TRY(hipSetDevice(s->device));
  if (n == 0) return CHM_OK;
  StreamGuard guard(s, hip_stream);
  std::vector<Job> jobs;
  jobs.push_back({strategy, 0, n, d_part_ranks, d_costs});
  return run_search(s, jobs, nullptr, nullptr, (hipStream_t)hip_stream);
}

extern "C" int chm_rank_partitions(chm_scenario *s, int32_t strategy, const uint8_t *d_cuts, uint64_t n,
                                   uint64_t *d_part_ranks, void *hip_stream) {
  if (!s || strategy < 0 || strategy > 2 || (n && (!d_cuts || !d_part_ranks))) return CHM_ERR_ARG;
  const chm_family *f = find_family(s, strategy);
  if (!f) return CHM_ERR_UNRECOVERABLE;
  HIP_TRY(hipSetDevice(s->device));
  StreamGuard guard(s, hip_stream);
  if (chmk_rank_cuts(s->d_scn, f->stages - 1, d_cuts, n, d_part_ranks, hip_stream)) return CHM_ERR_HIP;
  return CHM_OK;
}

extern "C" int chm_search_ranks(chm_scenario *s, int32_t strategy, const uint64_t *d_part_ranks, uint64_t n,
                                int64_t *d_costs, chm_best *out, uint64_t *position, void *hip_stream) {
  if (!s || !out || strategy < 0 || strategy > 2 || (n && !d_part_ranks)) return CHM_ERR_ARG;
  const chm_family *f = find_family(s, strategy);
  if (!f) { nothing_found(out); return CHM_ERR_UNRECOVERABLE; }
  if (position) *position = UINT64_MAX;
  std::vector<Job> jobs;
  if (n) jobs.push_back({strategy, 0, n, d_part_ranks, d_costs});
  StreamGuard guard(s, hip_stream);
  return guard.settled(run_search(s, jobs, out, position, (hipStream_t)hip_stream));
}

extern "C" int chm_search_cuts(chm_scenario *s, int32_t strategy, const uint8_t *d_cuts, uint64_t n,
                               int64_t *d_costs, chm_best *out, uint64_t *position, void *hip_stream) {
  if (!s || !out || strategy < 0 || strategy > 2 || (n && !d_cuts)) return CHM_ERR_ARG;
  const chm_family *f = find_family(s, strategy);
  if (!f) { nothing_found(out); return CHM_ERR_UNRECOVERABLE; }
  if (position) *position = UINT64_MAX;
  std::vector<Job> jobs;
  if (n) {
    Job j{strategy, 0, n, nullptr, d_costs};
    j.cuts = d_cuts;
    jobs.push_back(j);
  }
  StreamGuard guard(s, hip_stream);
  return guard.settled(run_search(s, jobs, out, position, (hipStream_t)hip_stream));
}

extern "C" int chm_search_best(chm_scenario *s, uint32_t strategy_mask, chm_best *out, void *hip_stream) {
  if (!s || !out) return CHM_ERR_ARG;
  std::vector<Job> jobs;
  for (int i = 0; i < s->space.n_families; ++i) {
    const chm_family &f = s->space.fam[i];
    if (strategy_mask & (1u << f.strategy)) jobs.push_back({f.strategy, 0, f.n_part, nullptr, nullptr});
  }
  if (jobs.empty()) { nothing_found(out); return CHM_ERR_UNRECOVERABLE; }
  StreamGuard guard(s, hip_stream);
  return guard.settled(run_search(s, jobs, out, nullptr, (hipStream_t)hip_stream));
}

extern "C" int chm_search_best_batch(chm_scenario *const *handles, int32_t n, uint32_t strategy_mask, chm_best *outs,
                                     int32_t *codes, void *hip_stream) {
  if (n < 0 || (n > 0 && (!handles || !outs || !codes))) return CHM_ERR_ARG;
  if (n == 0) return CHM_OK;
  std::vector<const chm_scenario *> seen(handles, handles + n);
  std::sort(seen.begin(), seen.end());
  for (int i = 0; i < n; ++i)
    if (!seen[i] || (i > 0 && seen[i] == seen[i - 1]) || seen[i]->device != seen[0]->device) return CHM_ERR_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  HIP_TRY(hipSetDevice(handles[0]->device));
  // a large batch runs on the library's side streams, which start behind the work already in the caller's stream
  // and which the caller's stream is made to wait for at the end (through the events of the first handle)
  SideStreams *side = n >= BATCH_MIN ? side_streams_of(handles[0]->device) : nullptr;
  if (side && !side_fork(handles[0], side, st)) return CHM_ERR_HIP;
  auto stream_of = [&](int i) { return side ? side->stream[i % SIDE_STREAMS] : st; };
  std::vector<char> pending(n, 0);
  // whatever way the call ends: the caller's stream waits for the side streams, and every handle whose result
  // is not final leaves the caller's stream marked as busy
  struct Wrap {
    chm_scenario *const *h; int32_t n; const int32_t *codes; hipStream_t st; SideStreams *side;
    bool join() {
      const bool ok = side ? side_join(h[0], side, st) : true;
      side = nullptr;
      return ok;
    }
    ~Wrap() {
      (void)join();
      for (int i = 0; i < n; ++i)
        if (codes[i] != CHM_OK && codes[i] != CHM_ERR_NO_FEASIBLE && codes[i] != CHM_ERR_UNRECOVERABLE) mark_in_flight(h[i], st);
    }
  } wrap{handles, n, codes, st, side};
  for (int i = 0; i < n; ++i) codes[i] = CHM_ERR_HIP;          // until the handle's search has been collected
  for (int i = 0; i < n; ++i) {
    chm_scenario *s = handles[i];
    std::vector<Job> jobs;
    for (int k = 0; k < s->space.n_families; ++k) {
      const chm_family &f = s->space.fam[k];
      if (strategy_mask & (1u << f.strategy)) jobs.push_back({f.strategy, 0, f.n_part, nullptr, nullptr});
    }
    if (jobs.empty()) { nothing_found(&outs[i]); codes[i] = CHM_ERR_UNRECOVERABLE; continue; }
    // searches that need the host between two of their passes (a bounded search that enumerates candidates) run
    // on their own; all others are launched now and collected after one wait for the whole batch
    if (s->bounded && any_enumerable(s, jobs)) { codes[i] = run_search(s, jobs, &outs[i], nullptr, stream_of(i)); continue; }
    s->fast.penalty_by_capacity = s->bounded != 0;
    if (s->bounded) {
      std::vector<Job> all = make_seeds(s, jobs);
      all.insert(all.end(), jobs.begin(), jobs.end());
      jobs.swap(all);
    }
    codes[i] = launch_jobs(s, jobs, true, stream_of(i), ~0ull, s->bounded != 0, false);
    if (codes[i] != CHM_OK) { nothing_found(&outs[i]); continue; }
    if (s->search->ctx.device_finish || s->search->ctx.empty) { pending[i] = 1; codes[i] = CHM_ERR_HIP; }
    else codes[i] = collect_jobs(s, &outs[i], nullptr, stream_of(i), false);
  }
  if (!wrap.join() || hipStreamSynchronize(st) != hipSuccess) return CHM_ERR_HIP;
  for (int i = 0; i < n; ++i)
    if (pending[i]) codes[i] = collect_jobs(handles[i], &outs[i], nullptr, stream_of(i), true);
  for (int i = 0; i < n; ++i)
    if (codes[i] == CHM_ERR_HIP || codes[i] == CHM_ERR_ARG) return codes[i];
  return CHM_OK;
}

// ---- chm_search_best_static: the same search with its device scratch in a fixed array --------------------------
// What chm_search_best keeps in buffers allocated at load (the argmin words and counters of the call, the
// winner's reroute ranks, its transition time) lives here in one file-scope device array, so the call itself
// allocates nothing.  Every device the library runs on holds its own copy of the array at its own address;
// host code reaches it only through the address hipGetSymbolAddress returns, looked up once per device.
enum {
  STATIC_KEY_WORDS = 8192,                                  // argmin words, counters and incumbent of one call
  STATIC_WINNER_AT = STATIC_KEY_WORDS,                      // DEV_MAX_AFF words: reroute ranks of the winner
  STATIC_XFER_AT = STATIC_WINNER_AT + DEV_MAX_AFF,          // 8 + DEV_MAX_S bytes: transition time / migration scheme
  STATIC_WORDS = STATIC_KEY_WORDS + 16                      // 65,664 bytes
};
static_assert(STATIC_XFER_AT + 1 + DEV_MAX_S / 8 <= STATIC_WORDS, "layout of the static scratch");
static __device__ __align__(256) uint64_t scratch[STATIC_WORDS];

namespace {
enum { STATIC_MAX_DEVICES = 64 };
std::mutex static_mutex;
uint64_t *static_ptr[STATIC_MAX_DEVICES] = {};

// device address of `scratch` on `device` (which must be current); null when the lookup fails
uint64_t *static_scratch(int device) {
  if (device < 0 || device >= STATIC_MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(static_mutex);
  if (!static_ptr[device]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    static_ptr[device] = (uint64_t *)p;
  }
  return static_ptr[device];
}
}  // namespace

extern "C" int chm_search_best_static(chm_scenario *s, uint32_t strategy_mask, chm_best *out, void *hip_stream) {
  if (!s || !out) return CHM_ERR_ARG;
  std::vector<Job> jobs;
  for (int i = 0; i < s->space.n_families; ++i) {
    const chm_family &f = s->space.fam[i];
    if (!(strategy_mask & (1u << f.strategy))) continue;
    // reroute spaces that are swept by kernels of their own need per-partition scratch (tens of MB)
    if (f.strategy == 2 && s->fast.usable[2] && s->fast.split) { nothing_found(out); return CHM_ERR_LIMIT; }
    jobs.push_back({f.strategy, 0, f.n_part, nullptr, nullptr});
  }
  if (jobs.empty()) { nothing_found(out); return CHM_ERR_UNRECOVERABLE; }
  HIP_TRY(hipSetDevice(s->device));
  uint64_t *base = static_scratch(s->device);
  if (!base) return CHM_ERR_HIP;
  // the handle's own buffers step aside for the call
  uint64_t *const own_slots = s->d_slots, *const own_winner = s->d_winner, *const own_xfer = s->d_xfer;
  const uint32_t own_words = s->slot_words;
  const uint32_t own_ready = s->slots_ready_for;
  s->slots_ready_for = 0;                            // the shared array is filled at the start of every call
  s->d_slots = base; s->slot_words = STATIC_KEY_WORDS;
  s->d_winner = base + STATIC_WINNER_AT;
  s->d_xfer = base + STATIC_XFER_AT;
  s->fast.penalty_by_capacity = false;
  StreamGuard guard(s, hip_stream);
  const int rc = guard.settled(run_jobs(s, jobs, out, nullptr, (hipStream_t)hip_stream, ~0ull, false));
  s->d_slots = own_slots; s->slot_words = own_words; s->d_winner = own_winner; s->d_xfer = own_xfer;
  s->slots_ready_for = own_ready;
  if (rc == CHM_ERR_LIMIT) nothing_found(out);
  return rc;
}

extern "C" int chm_search_range(chm_scenario *s, int32_t strategy, uint64_t part_first, uint64_t part_count,
                                chm_best *out, void *hip_stream) {
  if (!s || !out || strategy < 0 || strategy > 2) return CHM_ERR_ARG;
  const chm_family *f = find_family(s, strategy);
  if (!f) { nothing_found(out); return CHM_ERR_UNRECOVERABLE; }
  if (part_first > f->n_part || part_count > f->n_part - part_first) return CHM_ERR_RANGE;
  std::vector<Job> jobs;
  jobs.push_back({strategy, part_first, part_count, nullptr, nullptr});
  StreamGuard guard(s, hip_stream);
  return guard.settled(run_search(s, jobs, out, nullptr, (hipStream_t)hip_stream));
}

extern "C" int chm_transfer_plan(chm_scenario *s, uint64_t part_rank, int32_t pipeline, int32_t *n_nodes,
                                 uint8_t *node_stage, uint8_t *stage_of_node, int64_t *fetch_mib, void *hip_stream) {
  if (!s || !n_nodes || !node_stage || !stage_of_node || !fetch_mib) return CHM_ERR_ARG;
  const chm_family *f = find_family(s, 1);
  if (!f) return CHM_ERR_UNRECOVERABLE;
  if (pipeline < 0 || pipeline >= s->h.D) return CHM_ERR_ARG;
  const std::vector<uint8_t> &sv = s->survivors[pipeline];
  if ((int)sv.size() == s->h.S) return CHM_ERR_ARG;          // this pipeline lost nothing: it keeps its layout
  if (part_rank >= f->n_part) return CHM_ERR_RANGE;
  HIP_TRY(hipSetDevice(s->device));
  hipStream_t st = (hipStream_t)hip_stream;
  uint8_t *d_stage = (uint8_t *)(s->d_xfer + 1);
  StreamGuard guard(s, hip_stream);
  if (chmk_transfer_plan(s->d_scn, part_rank, (int32_t)sv.size(), sv.data(), d_stage, (int64_t *)s->d_xfer, st)) return CHM_ERR_HIP;
  HIP_TRY(hipMemcpyAsync(s->h_pinned, s->d_xfer, sizeof(uint64_t) + DEV_MAX_S, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  *n_nodes = (int32_t)sv.size();
  *fetch_mib = (int64_t)s->h_pinned[0];
  const uint8_t *got = (const uint8_t *)(s->h_pinned + 1);
  for (size_t i = 0; i < sv.size(); ++i) { node_stage[i] = sv[i]; stage_of_node[i] = got[i]; }
  return guard.settled(CHM_OK);
}

extern "C" int chm_decode_plan(const chm_scenario *s, uint64_t index, chm_best *out) {
  if (!s || !out) return CHM_ERR_ARG;
  if (index >= s->space.n_plans) return CHM_ERR_RANGE;
  for (int i = 0; i < s->space.n_families; ++i) {
    const chm_family &f = s->space.fam[i];
    if (index < f.offset || index >= f.offset + f.n_part * f.n_reroute) continue;
    const uint64_t local = index - f.offset;
    uint64_t joint = local % f.n_reroute, rr[DEV_MAX_AFF] = {};
    if (f.strategy == 2)
      for (int a = s->h.n_aff - 1; a >= 0; --a) { rr[a] = joint % s->h.aff_R[a]; joint /= s->h.aff_R[a]; }
    fill_plan(s, &f, local / f.n_reroute, rr, 0, out);
    return CHM_OK;
  }
  return CHM_ERR_RANGE;
}

extern "C" int chm_set_timing(chm_scenario *s, int32_t on) {
  if (!s) return CHM_ERR_ARG;
  s->timing = on != 0;
  return CHM_OK;
}

extern "C" int chm_set_filter_compaction(chm_scenario *s, int32_t mode, float *share) {
  if (!s || mode < -1 || mode > 1) return CHM_ERR_ARG;
  s->fast.queue_mode = mode;
  if (share)
    for (int k = 0; k < 3; ++k) share[k] = fast_fit_share(&s->fast, s->h, k);
  return CHM_OK;
}

extern "C" int chm_set_bounded_search(chm_scenario *s, int32_t on) {
  if (!s) return CHM_ERR_ARG;
  s->bounded = on == 2 ? 2 : (on != 0 ? 1 : 0);
  return CHM_OK;
}

extern "C" int chm_get_timing(const chm_scenario *s, chm_timing *out) {
  if (!s || !out) return CHM_ERR_ARG;
  *out = s->last;
  return CHM_OK;
}

extern "C" int chm_family_classes(const chm_scenario *s, int32_t strategy, int32_t *n, int32_t *length,
                                  int32_t *micro_batches) {
  if (!s || !n || !length || !micro_batches || strategy < 0 || strategy > 2) return CHM_ERR_ARG;
  if (!find_family(s, strategy)) return CHM_ERR_UNRECOVERABLE;
  const DevFamily &f = s->h.fam[strategy];
  *n = f.n_cls;
  for (int i = 0; i < f.n_cls; ++i) { length[i] = f.cls[i].n; micro_batches[i] = f.cls[i].M; }
  return CHM_OK;
}

extern "C" int chm_reroute_shape(const chm_scenario *s, int32_t *n_affected, int32_t *peers, uint64_t *n_vectors) {
  if (!s || !n_affected || !peers || !n_vectors) return CHM_ERR_ARG;
  *n_affected = s->h.n_aff;
  for (int a = 0; a < DEV_MAX_AFF; ++a) {
    peers[a] = a < s->h.n_aff ? s->h.aff_peers[a] : 0;
    n_vectors[a] = a < s->h.n_aff ? s->h.aff_R[a] : 0;
  }
  return CHM_OK;
}

extern "C" void chm_free_scenario(chm_scenario *s) { release(s); }

extern "C" const char *chm_strerror(int code) {
  switch (code) {
    case CHM_OK: return "ok";
    case CHM_ERR_ARG: return "invalid argument";
    case CHM_ERR_RANGE: return "plan range or rank outside the plan space";
    case CHM_ERR_OVERFLOW: return "plan count or cost bound too large";
    case CHM_ERR_UNRECOVERABLE: return "no requested strategy can recover this failure set";
    case CHM_ERR_NO_FEASIBLE: return "every plan exceeds the memory cap";
    case CHM_ERR_HIP: return "HIP call failed";
    case CHM_ERR_LIMIT: return "beyond the limits of the allocation-free entry point";
    default: return "unknown error";
  }
}
