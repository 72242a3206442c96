// Stage 1: top-k expert selection per token row (Algorithm 1 step 1, "Gate"; Top-K of Section 6.3).
//
// HBM-streaming kernel: every logit is read once, k indices are written per row, and the only
// arithmetic is fp32 comparison.  A row is held by LANES consecutive lanes (1, 2, 4, ... 64), VPL
// values per lane; the k winners are extracted one by one: each lane scans its own values in
// ascending expert index with a strict '>' (so the lowest index wins ties), then the lane winners
// are combined across the group with DPP exchanges using (value descending, index ascending).
// Extracted entries are replaced by -inf, which no finite logit can tie with.
#include "common.h"

#include <cfloat>
#include <climits>

namespace rs {

template <int LANES, int VPL, bool VEC4>
__device__ __forceinline__ int slot_index(int q, int j)
{
    if constexpr (VEC4) return 4 * (q + LANES * (j >> 2)) + (j & 3);   // lane holds whole float4s, interleaved over lanes
    else return q + LANES * j;                                         // element-interleaved
}

template <int OFF>
__device__ __forceinline__ void argmax_step(float &bv, int &bi)
{
    const float ov = xlane<OFF>(bv);
    const int oi = xlane<OFF>(bi);
    const bool take = (ov > bv) || (ov == bv && oi < bi);
    bv = take ? ov : bv;
    bi = take ? oi : bi;
}

template <int LANES>
__device__ __forceinline__ void group_argmax(float &bv, int &bi)
{
    if constexpr (LANES >= 2) argmax_step<1>(bv, bi);
    if constexpr (LANES >= 4) argmax_step<2>(bv, bi);
    if constexpr (LANES >= 8) argmax_step<4>(bv, bi);
    if constexpr (LANES >= 16) argmax_step<8>(bv, bi);
    if constexpr (LANES >= 32) argmax_step<16>(bv, bi);
    if constexpr (LANES >= 64) argmax_step<32>(bv, bi);
}

template <int LANES, int VPL, bool VEC4>
__global__ __launch_bounds__(256) void route_topk_kernel(const float *__restrict__ logits, int64_t rows, int E, int k,
                                                         int32_t *__restrict__ topk_idx)
{
    constexpr int ROWS_PER_BLOCK = 256 / LANES;
    const int q = threadIdx.x % LANES;
    const int64_t first = (int64_t)blockIdx.x * ROWS_PER_BLOCK + threadIdx.x / LANES;
    const int64_t stride = (int64_t)gridDim.x * ROWS_PER_BLOCK;
    // every lane of a wave runs the same number of iterations (the exchanges need all lanes)
    const int64_t iters = (rows - (int64_t)blockIdx.x * ROWS_PER_BLOCK + stride - 1) / stride;

    for (int64_t it = 0; it < iters; ++it) {
        const int64_t row = first + it * stride;
        const bool live = row < rows;
        float v[VPL];
        if constexpr (VEC4) {
#pragma unroll
            for (int c = 0; c < VPL / 4; ++c) {
                const int e0 = 4 * (q + LANES * c);
                float4 x = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
                if (live && e0 < E) x = *reinterpret_cast<const float4 *>(logits + row * E + e0);
                v[4 * c + 0] = x.x; v[4 * c + 1] = x.y; v[4 * c + 2] = x.z; v[4 * c + 3] = x.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < VPL; ++j) {
                const int e = q + LANES * j;
                v[j] = (live && e < E) ? logits[row * E + e] : -INFINITY;
            }
        }

        int keep0 = 0, keep1 = 0;   // LANES == 1, k == 2: both winners leave in one 8-byte store
        for (int sel = 0; sel < k; ++sel) {
            float bv = -INFINITY;
            int bi = INT_MAX;
#pragma unroll
            for (int j = 0; j < VPL; ++j) {
                const bool better = v[j] > bv;
                bv = better ? v[j] : bv;
                bi = better ? slot_index<LANES, VPL, VEC4>(q, j) : bi;
            }
            group_argmax<LANES>(bv, bi);
#pragma unroll
            for (int j = 0; j < VPL; ++j)
                v[j] = (slot_index<LANES, VPL, VEC4>(q, j) == bi) ? -INFINITY : v[j];
            if constexpr (LANES == 1) {
                if (k == 2) { if (sel == 0) keep0 = bi; else keep1 = bi; }
                else if (live) topk_idx[row * k + sel] = bi;
            } else {
                if (live && q == (sel % LANES)) topk_idx[row * k + sel] = bi;
            }
        }
        if constexpr (LANES == 1) {
            if (k == 2 && live) *reinterpret_cast<int2 *>(topk_idx + row * 2) = make_int2(keep0, keep1);
        }
    }
}

template <int LANES, int VPL>
static int launch_topk(const float *logits, int64_t rows, int E, int k, int32_t *out, hipStream_t st)
{
    constexpr int ROWS_PER_BLOCK = 256 / LANES;
    int64_t blocks = (rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    const int64_t cap = 256 * 64;   // enough resident waves for the whole chip; longer inputs loop
    if (blocks > cap) blocks = cap;
    const bool vec4 = (E % 4 == 0) && (reinterpret_cast<uintptr_t>(logits) % 16 == 0);
    if (vec4)
        hipLaunchKernelGGL((route_topk_kernel<LANES, VPL, true>), dim3((unsigned)blocks), dim3(256), 0, st, logits, rows, E, k, out);
    else
        hipLaunchKernelGGL((route_topk_kernel<LANES, VPL, false>), dim3((unsigned)blocks), dim3(256), 0, st, logits, rows, E, k, out);
    return launch_status();
}

}  // namespace rs

extern "C" int railsched_route_topk(const float *logits, int64_t rows, int32_t E, int32_t k, int32_t *topk_idx,
                                    void *stream)
{
    using namespace rs;
    if (rows < 0 || E < 1 || k < 1 || k > E) return RAILSCHED_ERR_INVALID_ARG;
    if (E > kMaxExperts) return RAILSCHED_ERR_UNSUPPORTED;
    if (rows == 0) return RAILSCHED_OK;
    if (!logits || !topk_idx) return RAILSCHED_ERR_NULL_PTR;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (E <= 4) return launch_topk<1, 4>(logits, rows, E, k, topk_idx, st);
    if (E <= 8) return launch_topk<1, 8>(logits, rows, E, k, topk_idx, st);
    if (E <= 16) return launch_topk<4, 4>(logits, rows, E, k, topk_idx, st);
    if (E <= 32) return launch_topk<8, 4>(logits, rows, E, k, topk_idx, st);
    if (E <= 64) return launch_topk<16, 4>(logits, rows, E, k, topk_idx, st);
    if (E <= 128) return launch_topk<32, 4>(logits, rows, E, k, topk_idx, st);
    if (E <= 256) return launch_topk<64, 4>(logits, rows, E, k, topk_idx, st);
    if (E <= 512) return launch_topk<64, 8>(logits, rows, E, k, topk_idx, st);
    return launch_topk<64, 16>(logits, rows, E, k, topk_idx, st);
}
