// Device-side pieces of the LPT allocation (Algorithm 2, initialisation and step 3) shared by the stage-4
// kernels and by the one-call scheduler of small batches: lane-group reductions, the closed form for
// periods of equal weights, and the one-instance-per-wavefront loop.
#pragma once

#include "common.h"

namespace rs {

constexpr int kBatch = 64;          // packed shape: chunks per period and instance
constexpr int kLptWaves = 4;        // wavefronts per workgroup

// Issue priority of a wavefront by the length of its chain against the mean over all instances (len and mean are
// wave-uniform).  All wavefronts of a launch are resident together and the launch lasts as long as its longest
// chain; with equal priorities that chain shares its SIMD's issue slots evenly with shorter ones, which then finish
// early and leave the SIMD to it - with a higher priority it runs at its own pace from the start.
__device__ __forceinline__ void prioritise_long_chain(int64_t len, int64_t mean)
{
    const int64_t l = __builtin_amdgcn_readfirstlane((int)(len >> 8)), m = __builtin_amdgcn_readfirstlane((int)(mean >> 8));
    if (l > 2 * m) __builtin_amdgcn_s_setprio(3);
    else if (2 * l > 3 * m) __builtin_amdgcn_s_setprio(2);
    else if (4 * l > 5 * m) __builtin_amdgcn_s_setprio(1);
}

template <int GW> struct GroupBits;
template <> struct GroupBits<4> { static constexpr int S = 2; };
template <> struct GroupBits<8> { static constexpr int S = 3; };
template <> struct GroupBits<16> { static constexpr int S = 4; };
template <> struct GroupBits<32> { static constexpr int S = 5; };
template <> struct GroupBits<64> { static constexpr int S = 6; };

template <int CTRL>
__device__ __forceinline__ unsigned dpp_mov(unsigned v)
{
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}

// min(v, v of the partner lane).  Every lane has a partner under the controls used here, so bound_ctrl changes
// nothing - but it frees the compiler from tying the destination to an "old" value, and the exchange folds
// into one v_min_u32 with a DPP operand and no register copy in front of it.
template <int CTRL>
__device__ __forceinline__ unsigned dpp_min(unsigned v)
{
    return min(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ unsigned dpp_max(unsigned v)
{
    return max(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false));
}

template <int GW>
__device__ __forceinline__ unsigned group_min_u32(unsigned v)
{
    v = dpp_min<0xB1>(v);                           // quad_perm [1,0,3,2]
    v = dpp_min<0x4E>(v);                           // quad_perm [2,3,0,1]
    if constexpr (GW >= 8) v = dpp_min<0x141>(v);   // row_half_mirror
    if constexpr (GW >= 16) v = dpp_min<0x140>(v);  // row_mirror
    if constexpr (GW >= 32) v = min(v, xlane<16>(v));
    if constexpr (GW >= 64) v = min(v, xlane<32>(v));
    return v;
}

template <int GW>
__device__ __forceinline__ unsigned group_max_u32(unsigned v)
{
    v = dpp_max<0xB1>(v);
    v = dpp_max<0x4E>(v);
    if constexpr (GW >= 8) v = dpp_max<0x141>(v);
    if constexpr (GW >= 16) v = dpp_max<0x140>(v);
    if constexpr (GW >= 32) v = max(v, xlane<16>(v));
    if constexpr (GW >= 64) v = max(v, xlane<32>(v));
    return v;
}

template <int OFF>
__device__ __forceinline__ void lexmin_step(unsigned &hi, unsigned &lo, unsigned &q)
{
    const unsigned ohi = xlane<OFF>(hi), olo = xlane<OFF>(lo), oq = xlane<OFF>(q);
    const bool take = (ohi < hi) || (ohi == hi && (olo < lo || (olo == lo && oq < q)));
    hi = take ? ohi : hi; lo = take ? olo : lo; q = take ? oq : q;
}

// rail index of the lexicographically smallest (load, rail) pair of the group
template <int GW>
__device__ __forceinline__ unsigned group_argmin_u64(unsigned long long load, unsigned q)
{
    unsigned hi = (unsigned)(load >> 32), lo = (unsigned)load;
    lexmin_step<1>(hi, lo, q);
    lexmin_step<2>(hi, lo, q);
    if constexpr (GW >= 8) lexmin_step<4>(hi, lo, q);
    if constexpr (GW >= 16) lexmin_step<8>(hi, lo, q);
    if constexpr (GW >= 32) lexmin_step<16>(hi, lo, q);
    if constexpr (GW >= 64) lexmin_step<32>(hi, lo, q);
    return q;
}

// f(value held by the lane whose in-group index is q ^ mask, mask) for every mask in 1..GW-1
template <int GW, int T, typename F>
__device__ __forceinline__ void partners_shfl(unsigned v, F &f)
{
    if constexpr (T < GW) { f((unsigned)__shfl_xor((int)v, T, GW), (unsigned)T); partners_shfl<GW, T + 1>(v, f); }
}
template <typename F>
__device__ __forceinline__ void partners_quad(unsigned x, unsigned mask, F &f)
{
    if (mask != 0) f(x, mask);
    f(dpp_mov<0xB1>(x), mask ^ 1u);                 // quad_perm [1,0,3,2]
    f(dpp_mov<0x4E>(x), mask ^ 2u);                 // quad_perm [2,3,0,1]
    f(dpp_mov<0x1B>(x), mask ^ 3u);                 // quad_perm [3,2,1,0]
}
template <int GW, typename F>
__device__ __forceinline__ void for_each_partner(unsigned v, F f)
{
    if constexpr (GW <= 16) {
        partners_quad(v, 0u, f);
        if constexpr (GW >= 8) partners_quad(dpp_mov<0x141>(v), 7u, f);            // row_half_mirror: q ^ 7
        if constexpr (GW >= 16) {
            const unsigned r = dpp_mov<0x140>(v);                                 // row_mirror: q ^ 15
            partners_quad(r, 15u, f);
            partners_quad(dpp_mov<0x141>(r), 8u, f);
        }
    } else {
        partners_shfl<GW, 1>(v, f);
    }
}

// Closed form for a period of P chunks of one weight w > 0 entered with max - min load < w: with every
// rail within w of the emptiest one, greedy assignment of equal weights visits the rails round after
// round in the fixed order "ascending (load, rail)" - each pick lifts the emptiest rail above all
// others by less than w.  So chunk i of the period goes to the rail of rank i mod N, and the rail of
// rank s receives floor(P/N) + (s < P mod N) chunks.  Returns this lane's rank; adds its share to key.
template <int GW>
__device__ __forceinline__ unsigned closed_period(unsigned &key, bool has_rail, unsigned w, unsigned per_rank, unsigned extra)
{
    unsigned rank = 0;
    const unsigned mine = key;
    for_each_partner<GW>(mine, [&](unsigned other, unsigned) { rank += other < mine ? 1u : 0u; });
    if (has_rail) key += (w * (per_rank + (rank < extra ? 1u : 0u))) << GroupBits<GW>::S;
    return rank;
}

// in-group index of the lane whose rank equals `want` (ranks of rail lanes are a permutation of 0..N-1)
template <int GW>
__device__ __forceinline__ unsigned rail_of_rank(unsigned rank, unsigned q, unsigned want)
{
    unsigned res = q;
    for_each_partner<GW>(rank, [&](unsigned other, unsigned mask) { res = (other == want) ? (q ^ mask) : res; });
    return res;
}

// ================================================================================ wide shape
// One instance per wavefront.  Every row of 16 lanes (the whole wavefront for N > 16) carries the N rail
// loads and runs the same step, so all 64 lanes know each decision; lane t keeps the decision for chunk t of
// the 64-chunk period, and weights reach the chain through v_readlane (a scalar broadcast).
//
// lpt_wide_body schedules the `len` chunks whose weights start at wsrc (rails to rdst) from rails that
// all hold `base` bytes, and leaves the final loads in S_row[0..N).  Called by a whole wavefront.
// `spare` points at one readable word in the same kind of memory as wsrc (lanes past the end load it).
constexpr int kWideDepth = 2;       // periods of 64 chunks in flight per wavefront

// The decisions of a period, one per step, collect in a shift register across the 64 lanes: every lane takes its
// upper neighbour's value and lane 63 takes the new one (a DPP wavefront shift with the new value as the "old"
// operand that lanes without a source keep), so after 64 steps lane t holds the decision of step t.  One
// instruction per step, beside the chain, where a compare of the lane index with t and a select took two.
__device__ __forceinline__ unsigned shift_in(unsigned reg, unsigned v)
{
    return (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)reg, 0x130, 0xF, 0xF, false);   // wave_shl:1
}

template <int GW> struct WideLimit {
    // packing limit: inside a period no delta exceeds (64 + 2) maximal weights, and the largest
    // packed key must stay below the all-ones key of lanes that hold no rail
    static constexpr unsigned value = (unsigned)((0xFFFFFFFFu >> GroupBits<GW>::S) / (unsigned)(64 + 2)) - 1u;
};

// ---------------------------------------------------------------------------------------------
// Sorted form.  The N packed keys (delta << S | rail, all different) are kept in ascending order across the first N
// lanes of a row of 16 (N <= 16; of the wavefront otherwise) - as their complements t = ~key, so the list descends and
// the lanes behind it, like the lane behind the end that DPP reads as zero, hold "nothing" = 0.  The rail that takes
// the next chunk is then always the one in lane 0, and the greedy step
//     j* = argmin LoadState,  LoadState[j*] += w
// is "take lane 0's entry, add w, put it back where it belongs": with y = t[0] - (w << S), the entry of lane r
// becomes the median of (t[r], t[r+1], y).  Two dependent instructions per step (the subtraction reads lane 0
// through DPP, v_med3_u32 re-sorts) where a min reduction over the lanes, a compare and a select need five, and six
// issued where those need eight: 16 ns per step on a wavefront alone against 22, 26 against 46 with two wavefronts on
// the SIMD.  With N <= 16 all four rows carry the same list, so every lane sees y, whose low bits are the chosen rail.
__device__ __forceinline__ unsigned umed3(unsigned a, unsigned b, unsigned c)
{
    unsigned r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
// ROW: the list lives in a row of 16 lanes (N <= 16; the wavefront's four rows carry copies); otherwise it spans the wavefront
// (N <= 64), its head comes through the scalar unit and a step costs 30 ns instead of 16 - still half the reduction form's 62.
template <bool ROW>
__device__ __forceinline__ unsigned list_head(unsigned v)          // the list's first entry
{
    if constexpr (ROW) return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x150, 0xF, 0xF, true);   // row_newbcast:0
    else return (unsigned)__builtin_amdgcn_readfirstlane((int)v);
}
template <bool ROW>
__device__ __forceinline__ unsigned list_next(unsigned v)          // the next lane's entry; zero behind the last lane of the row / wavefront
{
    if constexpr (ROW) return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x101, 0xF, 0xF, true);   // row_shl:1
    else return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x130, 0xF, 0xF, true);                  // wave_shl:1
}

constexpr int kSortedBlock = 16;    // steps between two looks at how many chunks are left
// kSortedBlock steps of a period.  wvS holds the period's weights, shifted past the rail bits, one per lane; the ones the block needs are
// read out into vector registers ahead of the chain (a scalar read consumed right away stalls the wavefront, step after step).
template <bool ROW, int T0>
__device__ __forceinline__ void sorted_steps(unsigned &t, unsigned &won, unsigned wvS)
{
    unsigned w[kSortedBlock];
#pragma unroll
    for (int j = 0; j < kSortedBlock; ++j) {
        w[j] = (unsigned)__builtin_amdgcn_readlane((int)wvS, T0 + j);
        asm volatile("" : "+v"(w[j]));              // into a vector register: the subtraction's other operand comes through DPP
    }
#pragma unroll
    for (int j = 0; j < kSortedBlock; ++j) {
        const unsigned y = list_head<ROW>(t) - w[j];
        const unsigned nb = list_next<ROW>(t);
        won = shift_in(won, y);
        t = umed3(t, nb, y);
    }
}
// steps T0 .. of a period, block by block, for as long as chunks are left
template <bool ROW, int T0>
__device__ __forceinline__ void sorted_blocks(unsigned &t, unsigned &won, unsigned wvS, int left)
{
    if constexpr (T0 < 64) {
        if (T0 < left) {                            // wave-uniform
            sorted_steps<ROW, T0>(t, won, wvS);
            sorted_blocks<ROW, T0 + kSortedBlock>(t, won, wvS, left);
        }
    }
}

template <int GW, bool RUNS>
__device__ __forceinline__ void lpt_wide_body_sorted(const uint32_t *__restrict__ wsrc, uint8_t *__restrict__ rdst, int64_t len,
                                                     unsigned long long base, int N, int64_t *__restrict__ S_row,
                                                     const uint32_t *__restrict__ spare)
{
    constexpr bool ROW = GW <= 16;
    constexpr int S = GroupBits<GW>::S;
    constexpr unsigned MASK = (unsigned)GW - 1u;
    constexpr int P = 64;                           // chunks per period: one per lane
    constexpr unsigned W_LIMIT = WideLimit<GW>::value;
    const int lane = threadIdx.x & 63;
    const unsigned r = ROW ? (unsigned)lane & 15u : (unsigned)lane;   // place in the list
    const bool in_list = (int)r < N;
    const unsigned q = (unsigned)(lane % GW);       // the exact path keeps loads by rail, lane q of a group of GW
    const bool has_rail = (int)q < N;

    unsigned t = in_list ? ~r : 0u;                 // all deltas 0: ascending rail index
    unsigned long long load = has_rail ? 0ull : ~0ull;
    bool exact = false;

    const unsigned per_rank = (unsigned)(P / N), extra = (unsigned)(P % N);
    const int place_of_chunk = lane % N;                                        // list place that takes chunk `lane` of a closed period
    const int after_closed = (ROW ? (lane & ~15) : 0) | (int)((r + extra) % (unsigned)N);   // lane whose entry moves here when the list rotates by `extra`

    // Weights move in requests of kWideDepth periods, as in the rail-indexed form above.
    auto weight_at = [&](int64_t i) { const uint32_t *src = (i < len) ? wsrc + i : spare; return *src; };
    unsigned cur[kWideDepth], nxt[kWideDepth], held[kWideDepth];
    auto store_rails = [&](int64_t i0) {
#pragma unroll
        for (int d = 0; d < kWideDepth; ++d) {
            const int64_t i = i0 + (int64_t)d * P + lane;
            if (i < len) rdst[i] = (uint8_t)held[d];
        }
    };
#pragma unroll
    for (int d = 0; d < kWideDepth; ++d) { nxt[d] = weight_at((int64_t)d * P + lane); held[d] = 0; }

    for (int64_t i0 = 0; i0 < len; i0 += (int64_t)kWideDepth * P) {
#pragma unroll
        for (int d = 0; d < kWideDepth; ++d) {
            asm volatile("" : "+v"(nxt[d]) : : "memory");                 // loads and stores below stay behind this wait
            cur[d] = nxt[d];
        }
#pragma unroll
        for (int d = 0; d < kWideDepth; ++d) nxt[d] = weight_at(i0 + (int64_t)(kWideDepth + d) * P + lane);
        if (i0 > 0) store_rails(i0 - (int64_t)kWideDepth * P);
#pragma unroll
        for (int d = 0; d < kWideDepth; ++d) {
            const int64_t p0 = i0 + (int64_t)d * P;
            if (p0 >= len) break;                   // wave-uniform
            const unsigned wv = (p0 + lane < len) ? cur[d] : 0u;
            unsigned won = 0;
            if (!exact && __ballot(wv > W_LIMIT) != 0ull) {
                // leave the packed keys for good: loads by rail, 64 bits each.  Lane q takes the entry of its rail.
                exact = true;
                for (int place = 0; place < N; ++place) {
                    const unsigned key = ~(unsigned)__builtin_amdgcn_readlane((int)t, place);
                    if (has_rail && (key & MASK) == q) load = base + (unsigned long long)(key >> S);
                }
            }
            bool closed = false;
            unsigned w0 = 0;
            if (RUNS && !exact) {
                w0 = (unsigned)__builtin_amdgcn_readfirstlane((int)wv);
                const unsigned dmin = (~(unsigned)__builtin_amdgcn_readfirstlane((int)t)) >> S;
                const unsigned dmax = (~(unsigned)__builtin_amdgcn_readlane((int)t, N - 1)) >> S;
                const bool ok = (wv == w0) && w0 != 0u && (p0 + P <= len) && (dmax - dmin) < w0;
                closed = __ballot(!ok) == 0ull;
            }
            if (closed) {
                // Equal weights from loads within one weight of each other: the list is visited front to back, round
                // after round (see closed_period), so chunk i goes to place i mod N, place s takes floor(P/N) + (s < P mod N)
                // chunks, and afterwards the places that took one chunk fewer come first, both parts in their old order:
                // the list rotated by P mod N.
                won = (~(unsigned)__shfl((int)t, place_of_chunk)) & MASK;
                const unsigned grown = t - ((w0 * (per_rank + (r < extra ? 1u : 0u))) << S);
                const unsigned moved = (unsigned)__shfl((int)grown, after_closed);
                t = in_list ? moved : 0u;
            } else if (!exact) {
                const int left = __builtin_amdgcn_readfirstlane((len - p0 < P) ? (int)(len - p0) : P);   // the last period stops where the chunks do
                sorted_blocks<ROW, 0>(t, won, wv << S, left);
                const int ran = (left + kSortedBlock - 1) & ~(kSortedBlock - 1);
                if (ran < P) won = (unsigned)__shfl((int)won, lane + (P - ran));   // a short period leaves step t in lane t + P - ran
                won = ~won & MASK;
            } else {
#pragma unroll 2
                for (int s = 0; s < P; ++s) {
                    const unsigned w = (unsigned)__builtin_amdgcn_readlane((int)wv, s);
                    const unsigned js = group_argmin_u64<GW>(load, q);
                    load += (q == js) ? (unsigned long long)w : 0ull;
                    won = shift_in(won, js);
                }
            }
            if (!exact) {
                // the emptiest rail's delta moves into the base, so deltas stay below the packing limit
                const unsigned adv = (~(unsigned)__builtin_amdgcn_readfirstlane((int)t)) >> S;
                if (in_list) t += adv << S;
                base += adv;
            }
            held[d] = won;
        }
    }
    if (len > 0) store_rails((len - 1) / ((int64_t)kWideDepth * P) * ((int64_t)kWideDepth * P));
    if (exact) {
        if (lane < N) S_row[lane] = (int64_t)load;
    } else if (lane < N) {
        const unsigned key = ~t;                    // row 0's list: place `lane` holds rail key & MASK
        S_row[key & MASK] = (int64_t)(base + (unsigned long long)(key >> S));
    }
}

template <int GW, bool RUNS>
__device__ __forceinline__ void lpt_wide_body(const uint32_t *__restrict__ wsrc, uint8_t *__restrict__ rdst, int64_t len,
                                              unsigned long long base, int N, int64_t *__restrict__ S_row,
                                              const uint32_t *__restrict__ spare)
{
    lpt_wide_body_sorted<GW, RUNS>(wsrc, rdst, len, base, N, S_row, spare);
}

}  // namespace rs
