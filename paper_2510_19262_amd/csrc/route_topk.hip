// Stage 1: top-k expert selection per token row (Algorithm 1 step 1, "Gate"; Top-K of Section 6.3).
//
// HBM-streaming kernel: every logit is read once, k indices are written per row, and the only
// arithmetic is fp32 comparison.  A row is held by LANES consecutive lanes (1, 2, 4, ... 64), VPL
// values per lane; the k winners are extracted one by one: each lane scans its own values in
// ascending expert index with a strict '>' (so the lowest index wins ties), then the lane winners
// are combined across the group with DPP exchanges using (value descending, index ascending).
// Extracted entries are replaced by -inf, which no finite logit can tie with.
#include "common.h"
#include "topk_core.h"

namespace rs {

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

// descending sort of 8 unique keys: Batcher's odd-even merge network, 19 exchanges
__device__ __forceinline__ void sort8_desc(unsigned (&a)[8])
{
    sort2_desc(a[0], a[1]); sort2_desc(a[2], a[3]); sort2_desc(a[4], a[5]); sort2_desc(a[6], a[7]);
    sort2_desc(a[0], a[2]); sort2_desc(a[1], a[3]); sort2_desc(a[4], a[6]); sort2_desc(a[5], a[7]);
    sort2_desc(a[1], a[2]); sort2_desc(a[5], a[6]);
    sort2_desc(a[0], a[4]); sort2_desc(a[1], a[5]); sort2_desc(a[2], a[6]); sort2_desc(a[3], a[7]);
    sort2_desc(a[2], a[4]); sort2_desc(a[3], a[5]);
    sort2_desc(a[1], a[2]); sort2_desc(a[3], a[4]); sort2_desc(a[5], a[6]);
}

// the 8 largest of two descending 8-lists, descending: max(a[i], b[7-i]) is that set as a bitonic sequence
__device__ __forceinline__ void top8_of_two(unsigned (&a)[8], const unsigned (&b)[8])
{
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = max(a[i], b[7 - i]);
    sort2_desc(a[0], a[4]); sort2_desc(a[1], a[5]); sort2_desc(a[2], a[6]); sort2_desc(a[3], a[7]);
    sort2_desc(a[0], a[2]); sort2_desc(a[1], a[3]); sort2_desc(a[4], a[6]); sort2_desc(a[5], a[7]);
    sort2_desc(a[0], a[1]); sort2_desc(a[2], a[3]); sort2_desc(a[4], a[5]); sort2_desc(a[6], a[7]);
}

// drop the head of a descending list held in registers (the winner's lane only)
template <int L, int J>
__device__ __forceinline__ void list_pop(unsigned (&lst)[8], bool win)
{
    if constexpr (J + 1 < L) {
        lst[J] = win ? lst[J + 1] : lst[J];
        list_pop<L, J + 1>(lst, win);
    } else {
        lst[J] = win ? 0u : lst[J];
    }
}

// LANES lanes per row, VPL logits per lane (VPL/4 float4 loads, interleaved over the lanes), a sorted list of
// L = min(VPL, 8) keys per lane: with k <= 8 a lane can never contribute more than its 8 best.  Fewer lanes per
// row mean fewer cross-lane steps per round and more rows per wavefront; the rounds dominate the instruction count.
template <int LANES, int VPL>
__global__ __launch_bounds__(256) void route_topk_keys_kernel(const float *__restrict__ logits, int64_t rows, int E, int k,
                                                              int32_t *__restrict__ topk_idx)
{
    constexpr int RPW = 64 / LANES;                 // rows per wavefront
    constexpr int NV = VPL / 4;                     // float4 loads per lane and row
    constexpr int L = VPL < 8 ? VPL : 8;            // sorted keys kept per lane
    constexpr unsigned MASK = (unsigned)(LANES * VPL) - 1u;   // expert index bits of a key
    static_assert(VPL == 4 || VPL == 8 || VPL == 16, "4, 8 or 16 logits per lane");
    const int lane = threadIdx.x & 63;
    const int q = lane % LANES;
    const int64_t wave_first = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW;
    const int64_t first = wave_first + lane / LANES;
    const int64_t stride = (int64_t)gridDim.x * 4 * RPW;
    const float4 none = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);

    float4 x[NV];
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const int e0 = 4 * (q + LANES * c);
        x[c] = (first < rows && e0 < E) ? load_stream4(logits + first * E + e0) : none;
    }
    for (int64_t w0 = wave_first; w0 < rows; w0 += stride) {            // wave-uniform trip count
        const int64_t row = first + (w0 - wave_first);
        const bool live = row < rows;
        float4 cur[NV];
        unsigned key[VPL];
#pragma unroll
        for (int c = 0; c < NV; ++c) {
            const int e0 = 4 * (q + LANES * c);
            const bool has = live && e0 < E;
            cur[c] = x[c];
            const int64_t nrow = row + stride;                          // next row, in flight while the rounds below run
            x[c] = (nrow < rows && e0 < E) ? load_stream4(logits + nrow * E + e0) : none;
            key[4 * c + 0] = has ? make_key<MASK>(cur[c].x, e0 + 0) : 0u; key[4 * c + 1] = has ? make_key<MASK>(cur[c].y, e0 + 1) : 0u;
            key[4 * c + 2] = has ? make_key<MASK>(cur[c].z, e0 + 2) : 0u; key[4 * c + 3] = has ? make_key<MASK>(cur[c].w, e0 + 3) : 0u;
        }
        unsigned lst[8];                                                // lst[0..L) descending, the lane's candidates
        if constexpr (VPL == 4) {
            sort2_desc(key[0], key[1]); sort2_desc(key[2], key[3]); sort2_desc(key[0], key[2]); sort2_desc(key[1], key[3]);
            sort2_desc(key[1], key[2]);
#pragma unroll
            for (int j = 0; j < 4; ++j) lst[j] = key[j];
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) lst[j] = key[j];
            sort8_desc(lst);
            if constexpr (VPL == 16) {
                unsigned hi[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) hi[j] = key[8 + j];
                sort8_desc(hi);
                top8_of_two(lst, hi);
            }
        }

        unsigned mine = 0, prev = 0;
        for (int sel = 0; sel < k; ++sel) {
            const unsigned K = group_max_all<LANES>(lst[0]);
            mine = (q == sel) ? K : mine;
            const bool win = (lst[0] == K);
            list_pop<L, 0>(lst, win);
            prev = K;
        }
        // the value cut is safe iff neighbouring winners, and the last winner and the best loser, differ above the index bits
        const unsigned up = (unsigned)__shfl_up((int)mine, 1);          // previous winner (lane q-1 of the same row)
        bool bad = (q >= 1 && q < k && ((mine ^ up) <= MASK)) || (lst[0] != 0u && ((lst[0] ^ prev) <= MASK));
        int result = (int)(MASK - (mine & MASK));
        if (__ballot(bad) != 0ull) {                                    // rare: full comparisons for this wavefront's rows
            float v[VPL];
#pragma unroll
            for (int c = 0; c < NV; ++c) {
                const bool has = live && 4 * (q + LANES * c) < E;
                v[4 * c + 0] = has ? cur[c].x : -INFINITY; v[4 * c + 1] = has ? cur[c].y : -INFINITY;
                v[4 * c + 2] = has ? cur[c].z : -INFINITY; v[4 * c + 3] = has ? cur[c].w : -INFINITY;
            }
            for (int sel = 0; sel < k; ++sel) {
                float bv = -INFINITY;
                int bi = INT_MAX;
#pragma unroll
                for (int j = 0; j < VPL; ++j) {
                    const bool better = v[j] > bv;
                    bv = better ? v[j] : bv;
                    bi = better ? slot_index<LANES, VPL, true>(q, j) : bi;
                }
                group_argmax<LANES>(bv, bi);
#pragma unroll
                for (int j = 0; j < VPL; ++j) v[j] = (slot_index<LANES, VPL, true>(q, j) == bi) ? -INFINITY : v[j];
                result = (q == sel) ? bi : result;
            }
        }
        if (live && q < k) topk_idx[row * k + q] = result;
    }
}

// WAVES: resident wavefronts per SIMD the register allocation is held to.
// FULL: E == LANES * VPL, every load is in range (rows beyond the last repeat the last row and are not stored).
template <int LANES, int VPL, int L, int WAVES, bool FULL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WAVES, 8))) void route_topk_insert_kernel(
    const float *__restrict__ logits, int64_t rows, int E, int k, int32_t *__restrict__ topk_idx, int wide_store)
{
    constexpr int RPW = 64 / LANES;                 // rows per wavefront
    constexpr unsigned MASK = (unsigned)(LANES * VPL) - 1u;   // expert index bits of a key
    const int lane = threadIdx.x & 63;
    const int q = lane % LANES;
    const int64_t row = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / LANES;   // one row group per wavefront
    const bool live = row < rows;

    float4 x[VPL / 4];
    row_load<LANES, VPL, FULL>(logits + (live ? row : rows - 1) * E, E, q, x);
    float own[L];
    lane_best<LANES, VPL, L>(x, q, own);
    unsigned u[8];
    const bool bad = row_best8<LANES, VPL, L>(own, k, u);
    if (__ballot(live && bad) == 0ull) {
        store_best8<LANES, MASK>(topk_idx, row, k, q, live, wide_store, u);
        return;
    }
    // rare: the wavefront's rows are read again and picked by full comparisons
    row_exact<LANES, VPL>(logits + row * E, live, E, k, q, [&](int sel, int bi) {
        if (live && q == sel % LANES) topk_idx[row * k + sel] = bi;
    });
}

template <int LANES, int VPL, int L, int WAVES>
static int launch_topk_insert(const float *logits, int64_t rows, int E, int k, int32_t *out, hipStream_t st)
{
    constexpr int ROWS_PER_BLOCK = 4 * (64 / LANES);
    const int64_t blocks = (rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    if (blocks > 0x7FFFFFFFll) return RAILSCHED_ERR_UNSUPPORTED;
    const int wide_store = reinterpret_cast<uintptr_t>(out) % 16 == 0 ? 1 : 0;
    if (E == LANES * VPL)
        hipLaunchKernelGGL((route_topk_insert_kernel<LANES, VPL, L, WAVES, true>), dim3((unsigned)blocks), dim3(256), 0, st, logits, rows, E, k, out, wide_store);
    else
        hipLaunchKernelGGL((route_topk_insert_kernel<LANES, VPL, L, WAVES, false>), dim3((unsigned)blocks), dim3(256), 0, st, logits, rows, E, k, out, wide_store);
    return launch_status();
}

template <int LANES, int VPL>
static int launch_topk_keys(const float *logits, int64_t rows, int E, int k, int32_t *out, hipStream_t st)
{
    constexpr int ROWS_PER_BLOCK = 4 * (64 / LANES);
    int64_t blocks = (rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL((route_topk_keys_kernel<LANES, VPL>), dim3((unsigned)blocks), dim3(256), 0, st, logits, rows, E, k, out);
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
    if (vec4 && E > 32 && E <= 64 && k <= 8) return launch_topk_insert<4, 16, 8, 6>(logits, rows, E, k, topk_idx, st);
    if (vec4 && E > 32 && E <= 64 && k <= 16) return launch_topk_keys<16, 4>(logits, rows, E, k, topk_idx, st);
    if (vec4 && E > 64 && E <= 128 && k <= 8) return launch_topk_insert<4, 32, 8, 6>(logits, rows, E, k, topk_idx, st);
    if (vec4 && E > 64 && E <= 128 && k <= 32) return launch_topk_keys<32, 4>(logits, rows, E, k, topk_idx, st);
    if (vec4 && E > 128 && E <= 256 && k <= 8) return launch_topk_insert<8, 32, 6, 5>(logits, rows, E, k, topk_idx, st);
    if (vec4 && E > 128 && E <= 256 && k <= 64) return launch_topk_keys<64, 4>(logits, rows, E, k, topk_idx, st);
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
