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

// Logits are read once and indices written once: streaming (non-temporal) accesses keep them from
// displacing anything useful in the caches.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float4 load_stream4(const float *p)
{
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream2(int32_t *p, int a, int b)
{
    i32x2 v; v.x = a; v.y = b;
    __builtin_nontemporal_store(v, reinterpret_cast<i32x2 *>(p));
}

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
                if (live && e0 < E) x = load_stream4(logits + row * E + e0);
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
            if (k == 2 && live) store_stream2(topk_idx + row * 2, keep0, keep1);
        }
    }
}


// ---------------------------------------------------------------------------------------------
// Packed-key variant for rows of 64..256 logits (LANES = 16, 32 or 64 lanes per row, one float4 each).
// Every logit becomes one 32-bit key: the upper bits are the order-preserving integer image of the
// float cut to 32 - IDXBITS bits, the low IDXBITS bits hold (MASK - expert index), so keys are unique,
// a plain unsigned max picks "largest value, lowest index", and one v_max_u32 per DPP step replaces
// the (value, index) pair exchange.  Each lane keeps its four keys sorted, so removing a winner is a
// shift.  Cutting the value is only safe when no two of the k winners, nor the last winner and the
// best loser, share a cut value; that is checked, and a row group that fails the check (two of its
// top logits within 2^-17 relative or closer) is redone with full (value, index) comparisons.
// ---------------------------------------------------------------------------------------------
template <int LANES>
__device__ __forceinline__ unsigned group_max_all(unsigned v)
{
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false));   // row_half_mirror
    v = max(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false));   // row_mirror
    if constexpr (LANES == 32) v = max(v, xlane<16>(v));
    if constexpr (LANES == 64) {
        v = max(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false));   // row_bcast15 into rows 1,3
        v = max(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false));   // row_bcast31 into rows 2,3
        v = (unsigned)__builtin_amdgcn_readlane((int)v, 63);
    }
    return v;
}

template <unsigned MASK>
__device__ __forceinline__ unsigned make_key(float f, unsigned idx)
{
    unsigned b = (unsigned)__float_as_int(f);
    b = (b == 0x80000000u) ? 0u : b;                                    // -0 ties with +0
    const unsigned ord = b ^ ((unsigned)((int)b >> 31) | 0x80000000u);  // monotone float -> unsigned
    return (ord & ~MASK) | (MASK - idx);
}

__device__ __forceinline__ void sort2_desc(unsigned &a, unsigned &b)
{
    const unsigned hi = max(a, b), lo = min(a, b);
    a = hi; b = lo;
}

template <int LANES>
__global__ __launch_bounds__(256) void route_topk_keys_kernel(const float *__restrict__ logits, int64_t rows, int E, int k,
                                                              int32_t *__restrict__ topk_idx)
{
    constexpr int RPW = 64 / LANES;                 // rows per wavefront
    constexpr unsigned MASK = 4u * LANES - 1u;      // expert index bits of a key
    const int lane = threadIdx.x & 63;
    const int q = lane % LANES;
    const int64_t first = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / LANES;
    const int64_t stride = (int64_t)gridDim.x * 4 * RPW;
    const int64_t wave_first = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW;
    const int e0 = 4 * q;
    const float4 none = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);

    float4 x = (first < rows && e0 < E) ? load_stream4(logits + first * E + e0) : none;
    for (int64_t w0 = wave_first; w0 < rows; w0 += stride) {            // wave-uniform trip count
        const int64_t row = first + (w0 - wave_first);
        const bool live = row < rows;
        const bool has = live && e0 < E;
        const float4 cur = x;
        {   // next row of this lane group, in flight while the rounds below run
            const int64_t nrow = row + stride;
            x = (nrow < rows && e0 < E) ? load_stream4(logits + nrow * E + e0) : none;
        }
        unsigned k0 = has ? make_key<MASK>(cur.x, e0 + 0) : 0u, k1 = has ? make_key<MASK>(cur.y, e0 + 1) : 0u;
        unsigned k2 = has ? make_key<MASK>(cur.z, e0 + 2) : 0u, k3 = has ? make_key<MASK>(cur.w, e0 + 3) : 0u;
        sort2_desc(k0, k1); sort2_desc(k2, k3); sort2_desc(k0, k2); sort2_desc(k1, k3); sort2_desc(k1, k2);

        unsigned mine = 0, prev = 0xFFFFFFFFu;
        bool bad = false;
        for (int sel = 0; sel < k; ++sel) {
            const unsigned K = group_max_all<LANES>(k0);
            bad = bad || ((prev ^ K) <= MASK);                          // two winners with the same cut value
            mine = (q == sel) ? K : mine;
            const bool win = (k0 == K);
            k0 = win ? k1 : k0; k1 = win ? k2 : k1; k2 = win ? k3 : k2; k3 = win ? 0u : k3;
            prev = K;
        }
        bad = bad || (k0 != 0u && ((k0 ^ prev) <= MASK));               // best loser against the last winner
        int result = (int)(MASK - (mine & MASK));

        if (__ballot(bad) != 0ull) {                                    // rare: full comparisons for this wavefront's rows
            float v[4] = {cur.x, cur.y, cur.z, cur.w};
            if (!has) { v[0] = v[1] = v[2] = v[3] = -INFINITY; }
            for (int sel = 0; sel < k; ++sel) {
                float bv = -INFINITY;
                int bi = INT_MAX;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool better = v[j] > bv;
                    bv = better ? v[j] : bv;
                    bi = better ? e0 + j : bi;
                }
                group_argmax<LANES>(bv, bi);
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = (e0 + j == bi) ? -INFINITY : v[j];
                result = (q == sel) ? bi : result;
            }
        }
        if (live && q < k) topk_idx[row * k + q] = result;
    }
}

template <int LANES>
static int launch_topk_keys(const float *logits, int64_t rows, int E, int k, int32_t *out, hipStream_t st)
{
    constexpr int ROWS_PER_BLOCK = 4 * (64 / LANES);
    int64_t blocks = (rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL((route_topk_keys_kernel<LANES>), dim3((unsigned)blocks), dim3(256), 0, st, logits, rows, E, k, out);
    return launch_status();
}

template <int LANES, int VPL>
static int launch_topk(const float *logits, int64_t rows, int E, int k, int32_t *out, hipStream_t st)
{
    constexpr int ROWS_PER_BLOCK = 256 / LANES;
    int64_t blocks = (rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    const int64_t cap = 1 << 22;    // one row group per thread measured fastest; only absurd sizes loop
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
    const bool vec4 = (E % 4 == 0) && (reinterpret_cast<uintptr_t>(logits) % 16 == 0);
    if (vec4 && E > 32 && E <= 64 && k <= 16) return launch_topk_keys<16>(logits, rows, E, k, topk_idx, st);
    if (vec4 && E > 64 && E <= 128 && k <= 32) return launch_topk_keys<32>(logits, rows, E, k, topk_idx, st);
    if (vec4 && E > 128 && E <= 256 && k <= 64) return launch_topk_keys<64>(logits, rows, E, k, topk_idx, st);
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
