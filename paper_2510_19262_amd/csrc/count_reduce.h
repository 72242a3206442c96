// Sum of the per-slice destination counts of stage 2 (Section 4.1, D^(1); Algorithm 1 step 2): slices of one
// (matrix, source GPU) pair leave their G counts side by side in a workspace, and
// D1[pair][d] = payload * sum over the pair's slices of count[pair][slice][d].  Defined in route_traffic.hip.
#pragma once

#include "common.h"

namespace rs {

// partial [n / G][splits][G] uint32 -> D1 [n] int64; n = pairs * G
int launch_count_reduce(const uint32_t *partial, int64_t *D1, int64_t n, int G, int splits, int64_t payload, hipStream_t st);

}  // namespace rs
