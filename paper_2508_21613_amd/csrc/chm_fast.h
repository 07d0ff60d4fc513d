// Shape-specialised search kernels (chm_fast.hip): interface to the host part.
#ifndef CHM_FAST_H
#define CHM_FAST_H
#include "chm_dev.h"

enum { FAST_MAX_P = 8, FAST_MAX_R = 4096 };

// One pipeline class in the form the specialised kernels read (all int32).
struct FastClass {
  int32_t n, M;
  int32_t dead0, dead1;           // partition stages missing from the chain (>= stages: none)
  int32_t unit;                   // 1: every node of the chain runs at nominal speed (no scaling)
  int32_t comm_total;             // (n-1) * comm
  uint32_t q[DEV_MAX_S];
  int32_t wlo[DEV_MAX_S], whi[DEV_MAX_S];   // memory prefix at the bounds of the fault-free stage of node j
};

struct FastFamily {
  int32_t n_cls;
  int32_t fixed_step;             // strategy 1: step time of the untouched pipelines
  int32_t w0[DEV_MAX_S + 1];      // memory prefix at the fault-free stage bounds
  int32_t w_total;                // memory of the whole model
  FastClass cls[DEV_MAX_CLS];
};

struct FastTables {
  FastFamily fam[3];
  // rerouting: per affected stage, all valid reroute vectors in rank order; a row has a stride of
  // 4 (up to 4 peers) or 8 dwords, and the row count is padded to a multiple of 4
  uint32_t vec_off[DEV_MAX_AFF];  // offset (in uint32) of stage a's rows in vecs[]
  uint32_t vec_rows[DEV_MAX_AFF]; // rows including the padding
};

struct FastState {
  bool usable[3] = {false, false, false};   // per strategy: a specialised kernel covers this scenario
  FastTables *d_tables = nullptr;
  uint32_t *d_vecs = nullptr;
};

// Decides per strategy whether a specialised kernel applies and uploads its tables.
// Returns 0, or non-zero on a failed HIP call.
int fast_prepare(FastState *f, const DevScenario &h, bool int32_ok);
// Launches the specialised search kernel for one chunk.  Returns 0 on success, a positive
// value when the strategy is not covered (the caller then uses the generic kernel), or a
// negative value on a HIP error.
int fast_search(FastState *f, const DevScenario &h, const SearchLaunch &a, void *stream);
void fast_release(FastState *f);
#endif
