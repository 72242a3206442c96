// Shared host/device helpers of the railsched library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "railsched.h"

namespace rs {

constexpr int kWave = 64;          // CDNA4 wavefront
constexpr int kMaxRails = 64;      // N: one rail per lane
constexpr int kMaxExperts = 1024;  // E
constexpr int kMaxGpus = 16384;    // G
constexpr int kMaxFlows = 16384;   // N*G flows of one (matrix, node) instance

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? RAILSCHED_OK : RAILSCHED_ERR_HIP;
}

// Host-side validation of the topology block shared by stages 2-5.
inline int check_topo(const railsched_topo_t *t)
{
    if (!t) return RAILSCHED_ERR_NULL_PTR;
    if (t->nodes < 1 || t->rails < 1 || t->chunk_bytes < 1 || t->reserved != 0) return RAILSCHED_ERR_INVALID_ARG;
    if (t->include_intra_node != 0 && t->include_intra_node != 1) return RAILSCHED_ERR_INVALID_ARG;
    if (t->rails > kMaxRails) return RAILSCHED_ERR_UNSUPPORTED;
    if ((int64_t)t->nodes * t->rails > kMaxGpus) return RAILSCHED_ERR_UNSUPPORTED;
    if (t->chunk_bytes > 0xFFFFFFFFll) return RAILSCHED_ERR_UNSUPPORTED;
    return RAILSCHED_OK;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline bool is_pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }

inline int ilog2(int64_t x)
{
    int s = 0;
    while ((int64_t(1) << (s + 1)) <= x) ++s;
    return s;
}

#if defined(__HIPCC__)
// ---- cross-lane exchange: lane i reads the lane that differs from it at "distance" OFF.
// 1 and 2 swap inside quads, 4 mirrors 8-lane halves, 8 mirrors 16-lane rows, 16 swaps rows through
// the LDS crossbar, 32 swaps wave halves.  After steps 1..OFF every group of 2*OFF lanes that
// combined a commutative, associative operation holds the same value in all its lanes.
template <int OFF>
__device__ __forceinline__ int xlane(int v)
{
    if constexpr (OFF == 1) return __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false);        // quad_perm [1,0,3,2]
    else if constexpr (OFF == 2) return __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
    else if constexpr (OFF == 4) return __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, false);  // row_half_mirror
    else if constexpr (OFF == 8) return __builtin_amdgcn_update_dpp(v, v, 0x140, 0xF, 0xF, false);  // row_mirror
    else if constexpr (OFF == 16) return __builtin_amdgcn_ds_swizzle(v, 0x401F);                    // lane ^ 16
    else return __builtin_amdgcn_ds_bpermute((int)(((threadIdx.x & 63u) ^ 32u) << 2), v);          // lane ^ 32
}
template <int OFF>
__device__ __forceinline__ unsigned xlane(unsigned v) { return (unsigned)xlane<OFF>((int)v); }
template <int OFF>
__device__ __forceinline__ float xlane(float v) { return __int_as_float(xlane<OFF>(__float_as_int(v))); }

// last i in [0,n) with v[i] <= x (v[0] <= x): plain binary search by one lane
template <typename T>
__device__ __forceinline__ int last_le(const T *v, int n, T x)
{
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (v[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// last i in [0,n) with v[i] <= x (v[0] <= x), searched 64 ways per step by the whole wavefront: lane l probes
// the l-th of 64 evenly spaced entries and the highest lane that still sees v <= x wins.  Two or three dependent
// memory round trips instead of log2(n); every lane of the wavefront must call it with the same arguments.
template <typename T>
__device__ __forceinline__ int wave_last_le(const T *v, int n, T x)
{
    const int lane = threadIdx.x & 63;
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int step = (hi - lo + 63) / 64;
        const int idx = lo + lane * step;
        const unsigned long long ok = __ballot(idx < hi && v[idx] <= x);   // a prefix of lanes; lane 0 always
        const int top = 63 - __clzll((long long)ok);
        lo = lo + top * step;
        hi = (lo + step < hi) ? lo + step : hi;
    }
    return lo;
}
#endif

}  // namespace rs
