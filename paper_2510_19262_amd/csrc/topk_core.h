// Device-side pieces of the gating decision (Algorithm 1 step 1; Top-K of Section 6.3) shared by stage 1 and by the
// one-pass routing call: streaming loads and stores, the (value, index) argmax of the exact path, and the sorted
// per-lane key lists of the insertion kernels.
#pragma once

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

// ---------------------------------------------------------------------------------------------
// Insertion kernels for k <= 8 and rows of 64..256 logits: no rounds and no sorting networks.
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

// This lane's VPL logits of the row at `row_logits` (LANES lanes per row, float4s interleaved over the lanes).
// FULL: E == LANES * VPL, every load is in range.
template <int LANES, int VPL, bool FULL>
__device__ __forceinline__ void row_load(const float *__restrict__ row_logits, int E, int q, float4 (&x)[VPL / 4])
{
    const float lowest = -FLT_MAX;                  // stands in for logits that do not exist (E < LANES * VPL)
#pragma unroll
    for (int c = 0; c < VPL / 4; ++c) {
        const int e0 = 4 * (q + LANES * c);
        if constexpr (FULL) x[c] = load_stream4(row_logits + e0);
        else x[c] = e0 < E ? load_stream4(row_logits + e0) : make_float4(lowest, lowest, lowest, lowest);
    }
}

// The L largest keys among this lane's logits, descending.  The logits are not needed afterwards.
template <int LANES, int VPL, int L>
__device__ __forceinline__ void lane_best(const float4 (&x)[VPL / 4], int q, float (&own)[L])
{
    constexpr unsigned MASK = (unsigned)(LANES * VPL) - 1u;   // expert index bits of a key
    static_assert(VPL % 4 == 0 && VPL >= 8 && LANES >= 2 && LANES <= 16 && L >= 4 && L <= 8 && L <= VPL, "shape");
    insert_loaded<LANES, VPL, L, MASK, 0, 0>(x, ~MASK | (unsigned)(4 * q), own);
}

// The 8 largest keys of the row from the lists of its LANES lanes, as bit patterns in u[0..8), the same in all lanes of the
// row.  Returns true when the result cannot be trusted (see above): the caller then picks the row's winners by full comparisons.
template <int LANES, int VPL, int L>
__device__ __forceinline__ bool row_best8(const float (&own)[L], int k, unsigned (&u)[8])
{
    constexpr unsigned MASK = (unsigned)(LANES * VPL) - 1u;
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
    return close < MASK || own[L - 1] >= kth;       // ... or every key this lane kept is a winner
}

// expert indices of the row's k winners to topk_idx[row][0..k)
template <int LANES, unsigned MASK>
__device__ __forceinline__ void store_best8(int32_t *__restrict__ topk_idx, int64_t row, int k, int q, bool live, int wide_store,
                                            const unsigned (&u)[8])
{
    if (wide_store && k == 8) {                     // one lane stores the row's eight indices: two 16-byte stores
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
}

// The k winners of the row by full (value, index) comparisons, one round each: emit(j, expert) is called in every lane
// of the row for j = 0 .. k-1.  Lanes of rows that do not exist (live == false) load nothing and take part in the exchanges.
template <int LANES, int VPL, typename F>
__device__ __forceinline__ void row_exact(const float *__restrict__ row_logits, bool live, int E, int k, int q, F emit)
{
    float v[VPL];
#pragma unroll
    for (int c = 0; c < VPL / 4; ++c) {
        const int e0 = 4 * (q + LANES * c);
        const float4 cur = (live && e0 < E) ? load_stream4(row_logits + e0) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
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
        emit(sel, bi);
    }
}

}  // namespace rs
