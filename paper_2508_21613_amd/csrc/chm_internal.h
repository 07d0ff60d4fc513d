// Entry points shared between the translation units of libchm that are not part of the C-ABI.
#ifndef CHM_INTERNAL_H
#define CHM_INTERNAL_H
#include <stdint.h>

#include "../../include/chm.h"
#include "../../include/chm_measure.h"

// A scenario holding one stand-alone pipeline of n stages and M micro-batches on identical nodes:
// its only family is strategy 1, a plan's cost is the pipeline's 1F1B time + comm per stage boundary.
int chm_internal_load_pipeline(int32_t L, const int32_t *fwd_us, const int32_t *bwd_us, const int32_t *mem_mib,
                               const int32_t *act_mib, int32_t n, int32_t M, int32_t comm_us, int32_t mem_cap_mib,
                               chm_scenario **out);
// micro-batches over pipelines in proportion to their node counts (Planner, "Batch Distribution")
void chm_internal_share_micro_batches(int D, int total, const int *nodes, int *out);
#endif
