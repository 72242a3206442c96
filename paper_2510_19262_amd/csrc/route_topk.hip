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
typedef int i32x4 __attribute__((ext_vector_type(4)));
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

// ---------------------------------------------------------------------------------------------
// Insertion variant for k <= 8 and rows of 64..256 logits: no rounds and no sorting networks.
//
// Keys are floats.  A logit keeps its sign, exponent and upper mantissa bits and takes its expert index into the
// low IDXBITS bits of the mantissa, so every key of a row is a different finite float, ordinary float comparison
// orders keys by their "cut" value, and the index comes back with one AND.  (-0 becomes +0 first, by adding +0.)
// The index bits are never trusted to order two logits of the same cut value: such rows are found and redone
// exactly, see below.  Two instructions per logit.
// A lane keeps the L largest keys it has seen as a descending list in registers.  Inserting x into a >= b >= c...
// is one instruction per entry: the new i-th entry is the median of (old entry i-1, old entry i, x), the new head
// max(head, x).  Then the LANES lanes of a row merge pairwise, log2(LANES) times, each keeping the 8 largest of
// its own and its partner's list (max(a[i], b[7-i]) is that set as a bitonic sequence; three exchange layers sort
// it); both partners end with the same list, so finally every lane of the row holds the row's 8 largest keys.
// The result is exact unless (a) two of those 8, or the k-th winner and a key that lost, share a cut value, or
// (b) a lane's whole list ended up among the winners, so that a key it dropped might have belonged there too (or
// be the best loser).  Both are tested on L + 8 registers; a wavefront with such a row re-reads its rows and picks
// by full (value, index) comparisons - rows full of exact ties take that path, continuous logits almost never do.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float fmed3(float a, float b, float c) { return __builtin_amdgcn_fmed3f(a, b, c); }

// x into the descending list a[0..HAVE) (a[0..L) once it is full)
template <int L, int HAVE>
__device__ __forceinline__ void list_insert(float (&a)[L], float x)
{
    if constexpr (HAVE == 0) {
        a[0] = x;
    } else {
        if constexpr (HAVE < L) a[HAVE] = fminf(a[HAVE - 1], x);
#pragma unroll
        for (int i = (HAVE < L ? HAVE - 1 : L - 1); i >= 1; --i) a[i] = fmed3(a[i - 1], a[i], x);   // old a[i-1]: bottom first
        a[0] = fmaxf(a[0], x);
    }
}

__device__ __forceinline__ void fsort2_desc(float &a, float &b)
{
    const float hi = fmaxf(a, b), lo = fminf(a, b);
    a = hi; b = lo;
}

// a bitonic sequence of 8 into descending order
__device__ __forceinline__ void bitonic8_desc(float (&a)[8])
{
    fsort2_desc(a[0], a[4]); fsort2_desc(a[1], a[5]); fsort2_desc(a[2], a[6]); fsort2_desc(a[3], a[7]);
    fsort2_desc(a[0], a[2]); fsort2_desc(a[1], a[3]); fsort2_desc(a[4], a[6]); fsort2_desc(a[5], a[7]);
    fsort2_desc(a[0], a[1]); fsort2_desc(a[2], a[3]); fsort2_desc(a[4], a[5]); fsort2_desc(a[6], a[7]);
}

template <int OFF>
__device__ __forceinline__ float from_partner(float v)
{
    constexpr int CTRL = OFF == 1 ? 0xB1 : OFF == 2 ? 0x4E : OFF == 4 ? 0x141 : 0x140;
    return __uint_as_float((unsigned)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), CTRL, 0xF, 0xF, true));
}

// the 8 largest of this lane's and its partner's descending lists of LEN entries (entries LEN..7 count as lowest);
// both partners end with the same list
template <int OFF, int LEN>
__device__ __forceinline__ void merge_lists(const float (&a)[LEN], float (&out)[8])
{
    static_assert(OFF == 1 || OFF == 2 || OFF == 4 || OFF == 8, "exchanges inside a row of 16 lanes");
    static_assert(LEN >= 4 && LEN <= 8, "lists of 4..8 keys");
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (i < 8 - LEN) out[i] = a[i];                               // the partner has nothing to set against it
        else if (i >= LEN) out[i] = from_partner<OFF>(a[7 - i]);     // nor this lane against the partner's
        else out[i] = fmaxf(a[i], from_partner<OFF>(a[7 - i]));      // folds into one v_max_f32 with a DPP operand
    }
    bitonic8_desc(out);
}

// key of a logit: cut value in the upper bits, expert index below.  lane_field has ones above the index bits and
// the lane's share of the index inside them; SLOT (a constant) likewise with the slot's share; the two never
// have an index bit in common.  One bit operation: (v & lane & slot) | (lane ^ slot).
template <unsigned SLOT>
__device__ __forceinline__ float make_fkey(float f, unsigned lane_field)
{
    return __uint_as_float(__builtin_amdgcn_bitop3_b32(__float_as_uint(f + 0.0f), lane_field, SLOT, 0xE6));
}

template <int LANES, int VPL, int L, unsigned MASK, int C, int J>
__device__ __forceinline__ void insert_loaded(const float4 (&x)[VPL / 4], unsigned lane_field, float (&lst)[L])
{
    if constexpr (C < VPL / 4) {
        constexpr unsigned SLOT = ~MASK | (unsigned)(4 * LANES * C + J);
        const float v = J == 0 ? x[C].x : J == 1 ? x[C].y : J == 2 ? x[C].z : x[C].w;
        list_insert<L, (4 * C + J < L ? 4 * C + J : L)>(lst, make_fkey<SLOT>(v, lane_field));
        insert_loaded<LANES, VPL, L, MASK, (J == 3 ? C + 1 : C), (J == 3 ? 0 : J + 1)>(x, lane_field, lst);
    }
}

// smallest of (a ^ b) - 1 and m: zero-based distance of two keys' bit patterns, all-ones when they are the same key
__device__ __forceinline__ unsigned min_xor_dist(unsigned m, unsigned a, unsigned b)
{
    return min(m, (a ^ b) - 1u);
}

// WAVES: resident wavefronts per SIMD the register allocation is held to.
// FULL: E == LANES * VPL, every load is in range (rows beyond the last repeat the last row and are not stored).
template <int LANES, int VPL, int L, int WAVES, bool FULL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WAVES, 8))) void route_topk_insert_kernel(
    const float *__restrict__ logits, int64_t rows, int E, int k, int32_t *__restrict__ topk_idx, int wide_store)
{
    constexpr int RPW = 64 / LANES;                 // rows per wavefront
    constexpr int NV = VPL / 4;                     // float4 loads per lane and row
    constexpr unsigned MASK = (unsigned)(LANES * VPL) - 1u;   // expert index bits of a key
    static_assert(VPL % 4 == 0 && VPL >= 8 && LANES >= 2 && LANES <= 16 && L >= 4 && L <= 8 && L <= VPL, "shape");
    const int lane = threadIdx.x & 63;
    const int q = lane % LANES;
    const int64_t row = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / LANES;   // one row group per wavefront
    const bool live = row < rows;
    const int64_t lrow = live ? row : rows - 1;
    const float lowest = -FLT_MAX;                  // stands in for logits that do not exist (E < LANES * VPL)

    float4 x[NV];
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const int e0 = 4 * (q + LANES * c);
        if constexpr (FULL) x[c] = load_stream4(logits + lrow * E + e0);
        else x[c] = e0 < E ? load_stream4(logits + lrow * E + e0) : make_float4(lowest, lowest, lowest, lowest);
    }
    float own[L];                                   // descending: the lane's L largest keys
    insert_loaded<LANES, VPL, L, MASK, 0, 0>(x, ~MASK | (unsigned)(4 * q), own);

    float lst[8];
    merge_lists<1, L>(own, lst);
    if constexpr (LANES >= 4) { float t[8]; merge_lists<2, 8>(lst, t);
#pragma unroll
        for (int i = 0; i < 8; ++i) lst[i] = t[i]; }
    if constexpr (LANES >= 8) { float t[8]; merge_lists<4, 8>(lst, t);
#pragma unroll
        for (int i = 0; i < 8; ++i) lst[i] = t[i]; }
    if constexpr (LANES >= 16) { float t[8]; merge_lists<8, 8>(lst, t);
#pragma unroll
        for (int i = 0; i < 8; ++i) lst[i] = t[i]; }

    // lst[j] = j-th largest key of the row (if no lane dropped one of them), the same in all its lanes
    unsigned u[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) u[j] = __float_as_uint(lst[j]);
    const float kth = k >= 8 ? lst[7] : k == 7 ? lst[6] : k == 6 ? lst[5] : k == 5 ? lst[4] : k == 4 ? lst[3] : k == 3 ? lst[2]
                    : k == 2 ? lst[1] : lst[0];
    const unsigned ukth = __float_as_uint(kth);
    unsigned close = 0xFFFFFFFFu;                   // (a ^ b) - 1 < MASK: a and b are different keys of one cut value
#pragma unroll
    for (int j = 1; j < 8; ++j) close = min_xor_dist(close, u[j], u[j - 1]);                  // neighbours among the row's best 8
#pragma unroll
    for (int i = 0; i < L; ++i) close = min_xor_dist(close, __float_as_uint(own[i]), ukth);   // this lane's keys against the k-th winner
    const bool bad = live && (close < MASK || own[L - 1] >= kth);      // ... or every key this lane kept is a winner

    if (__ballot(bad) == 0ull) {
        if (wide_store && k == 8) {                 // one lane stores the row's eight indices: two 16-byte stores
            if (live && q == 0) {
                i32x4 lo, hi;
                lo.x = (int)(u[0] & MASK); lo.y = (int)(u[1] & MASK); lo.z = (int)(u[2] & MASK); lo.w = (int)(u[3] & MASK);
                hi.x = (int)(u[4] & MASK); hi.y = (int)(u[5] & MASK); hi.z = (int)(u[6] & MASK); hi.w = (int)(u[7] & MASK);
                i32x4 *dst = reinterpret_cast<i32x4 *>(topk_idx + row * 8);
                __builtin_nontemporal_store(lo, dst);
                __builtin_nontemporal_store(hi, dst + 1);
            }
        } else {
#pragma unroll
            for (int r = 0; r < (8 + LANES - 1) / LANES; ++r) {          // winners q, q+LANES, ... of this lane
                unsigned sel = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) sel = (j == q + r * LANES) ? u[j] : sel;
                if (live && q + r * LANES < k) topk_idx[row * k + q + r * LANES] = (int)(sel & MASK);
            }
        }
        return;
    }
    // rare: the wavefront's rows are read again and picked by full comparisons
    float v[VPL];
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const int e0 = 4 * (q + LANES * c);
        const float4 cur = (live && e0 < E) ? load_stream4(logits + row * E + e0) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        v[4 * c + 0] = cur.x; v[4 * c + 1] = cur.y; v[4 * c + 2] = cur.z; v[4 * c + 3] = cur.w;
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
        if (live && q == sel % LANES) topk_idx[row * k + sel] = bi;
    }
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
