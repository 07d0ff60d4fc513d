// Shape-specialised search kernels (chm_fast.hip): interface to the host part.
#ifndef CHM_FAST_H
#define CHM_FAST_H
#include "chm_dev.h"

struct FastState {
  bool usable[3] = {false, false, false};   // per strategy: a specialised kernel covers this scenario
  void *d_tables = nullptr;                 // device block with the int32 tables those kernels read
};

// Decides per strategy whether a specialised kernel applies and uploads its tables.
// Returns 0, or a hipError_t on a failed HIP call.
int fast_prepare(FastState *f, const DevScenario &h, bool int32_ok);
// Launches the specialised search kernel for one chunk.  Returns 0 on success, a positive
// value when the strategy is not covered (the caller then uses the generic kernel), or a
// negative value on a HIP error.
int fast_search(FastState *f, const DevScenario &h, const SearchLaunch &a, void *stream);
void fast_release(FastState *f);
#endif
