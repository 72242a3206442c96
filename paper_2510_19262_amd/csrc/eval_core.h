// Argument block and the cross-file entry of the stage-5 reduction (Section 4.1 load matrices S and R;
// Theorem 2; Theorem 3), shared with the one-call scheduler of small batches.
#pragma once

#include "common.h"

namespace rs {

constexpr int kEvThreads = 256;

struct EvArgs {
    const int64_t *chunk_off;
    const uint32_t *chunk_w, *chunk_flow;
    const uint8_t *rail;
    const int64_t *S;
    int64_t *R, *stats;
    int64_t *partial;        // [batch][slices][G + 1]
    int32_t M, N, G, slices;
    int32_t nshift, gmask;   // >= 0 when N / G are powers of two
    int32_t wide_ok;         // record arrays aligned for 16-byte (weights, flows) and 4-byte (rails) loads
    int32_t copies;          // LDS copies of the receive bins (power of two); lanes that would add to one bin use different ones
    int64_t capacity;        // records the per-chunk arrays hold; more chunks than that: R and stats become -1
    int32_t n_inst;          // batch * M
};

__device__ __forceinline__ int dst_node(const EvArgs &a, uint32_t flow)
{
    // flow = n*G + dst  ->  dst / N
    if (a.gmask >= 0 && a.nshift >= 0) return (int)((flow & (uint32_t)a.gmask) >> a.nshift);
    return (int)((flow % (uint32_t)a.G) / (uint32_t)a.N);
}

// one workgroup per matrix: R = sum of the matrix's workspace slots, then the statistics (defined in eval.hip)
int launch_eval_reduce(const EvArgs &a, int batch, hipStream_t st);

}  // namespace rs
