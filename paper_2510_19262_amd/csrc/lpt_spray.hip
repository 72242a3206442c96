// Stage 4: LPT iterative allocation (Algorithm 2, initialisation and step 3).
//
// The loop is serial inside one (matrix, node) instance - every decision depends on all earlier
// ones - and independent across instances.  LoadState lives in lanes: a group of GW = 2^S lanes
// (GW >= N) holds one instance, lane q holds rail q, and 64/GW instances share a wavefront, so one
// instruction stream advances 64/GW schedulers.  Per chunk the group needs
//   j* = lowest-numbered rail of minimum load,   LoadState[j*] += w.
//
// Fast path.  Greedy assignment keeps max(LoadState) - min(LoadState) <= the largest weight seen so
// far (the fullest rail was the emptiest one just before its last chunk).  Loads are therefore kept
// as a 64-bit base shared by the group plus a small per-lane delta, and the lane packs
// key = (delta << S) | q into 32 bits: one unsigned min over the group, done with DPP exchanges,
// yields both the minimum and the lowest rail index that attains it, and key equality marks the
// winner.  The base is advanced every kBatch chunks so deltas stay small.
// Exact path.  As soon as a weight above the packing limit shows up, the instance group's wave
// switches for good to plain 64-bit loads with an explicit (load, rail) lexicographic reduction.
// Both paths compute the same function; the loads that leave the kernel are exact 64-bit sums.
#include "common.h"

namespace rs {

constexpr int kBatch = 32;          // chunks per normalisation period and instance (64 when a group is a whole wave)
constexpr int kLptWaves = 4;        // wavefronts per workgroup

template <int GW> struct GroupBits;
template <> struct GroupBits<4> { static constexpr int S = 2; };
template <> struct GroupBits<8> { static constexpr int S = 3; };
template <> struct GroupBits<16> { static constexpr int S = 4; };
template <> struct GroupBits<32> { static constexpr int S = 5; };
template <> struct GroupBits<64> { static constexpr int S = 6; };

template <int GW>
__device__ __forceinline__ unsigned group_min_u32(unsigned v)
{
    v = min(v, xlane<1>(v));
    v = min(v, xlane<2>(v));
    if constexpr (GW >= 8) v = min(v, xlane<4>(v));
    if constexpr (GW >= 16) v = min(v, xlane<8>(v));
    if constexpr (GW >= 32) v = min(v, xlane<16>(v));
    if constexpr (GW >= 64) v = min(v, xlane<32>(v));
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

// value held by lane T of the caller's GW-lane group
template <int GW, int T>
__device__ __forceinline__ unsigned group_bcast(unsigned v)
{
    if constexpr (GW == 64) return (unsigned)__builtin_amdgcn_readlane((int)v, T);
    else return (unsigned)__builtin_amdgcn_ds_swizzle((int)v, ((0x1F & ~(GW - 1)) | (T << 5)));   // lane = (lane & ~(GW-1)) | T
}

template <int GW, int STEP, int T>
__device__ __forceinline__ void fast_steps(unsigned &key, const unsigned (&wv)[STEP / GW], unsigned (&won)[STEP / GW], unsigned q)
{
    // chunk T of the period: its weight sits in lane T % GW of register T / GW
    if constexpr (T < STEP) {
        constexpr int S = GroupBits<GW>::S;
        const unsigned wS = group_bcast<GW, T % GW>(wv[T / GW]) << S;
        const unsigned m = group_min_u32<GW>(key);
        key += (key == m) ? wS : 0u;
        won[T / GW] = (q == (unsigned)(T % GW)) ? m : won[T / GW];
        fast_steps<GW, STEP, T + 1>(key, wv, won, q);
    }
}

template <int GW, int STEP, int T>
__device__ __forceinline__ void exact_steps(unsigned long long &load, const unsigned (&wv)[STEP / GW], unsigned (&won)[STEP / GW],
                                            unsigned q)
{
    if constexpr (T < STEP) {
        const unsigned w = group_bcast<GW, T % GW>(wv[T / GW]);
        const unsigned js = group_argmin_u64<GW>(load, q);
        load += (q == js) ? (unsigned long long)w : 0ull;
        won[T / GW] = (q == (unsigned)(T % GW)) ? js : won[T / GW];
        exact_steps<GW, STEP, T + 1>(load, wv, won, q);
    }
}

template <int GW>
__global__ __launch_bounds__(64 * kLptWaves) void lpt_spray_kernel(const int64_t *__restrict__ chunk_off,
                                                                   const uint32_t *__restrict__ chunk_w, int n_inst, int N,
                                                                   uint8_t *__restrict__ rail, int64_t *__restrict__ S_out)
{
    constexpr int S = GroupBits<GW>::S;
    constexpr int IPW = 64 / GW;                    // instances per wavefront
    constexpr int STEP = kBatch > GW ? kBatch : GW; // chunks per instance and normalisation period
    constexpr int REGS = STEP / GW;
    // packing limit: inside a period no delta exceeds (STEP + 2) maximal weights, and the largest
    // packed key must stay below the all-ones key of lanes that hold no rail
    constexpr unsigned W_LIMIT = (unsigned)((0xFFFFFFFFu >> S) / (unsigned)(STEP + 2)) - 1u;

    const int lane = threadIdx.x & 63;
    const unsigned q = (unsigned)(lane % GW);
    const int wave = (int)((blockIdx.x * (unsigned)kLptWaves) + (threadIdx.x >> 6));
    const int inst = wave * IPW + lane / GW;
    const bool has_inst = inst < n_inst;
    const bool has_rail = has_inst && (int)q < N;
    const int64_t beg = has_inst ? chunk_off[inst] : 0;
    const int64_t len = has_inst ? chunk_off[inst + 1] - beg : 0;

    int64_t max_len = len;                          // the wave runs as long as its longest instance
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) { const int64_t o = __shfl_xor(max_len, d); max_len = o > max_len ? o : max_len; }

    unsigned key = has_rail ? q : 0xFFFFFFFFu;
    unsigned long long base = 0, load = has_rail ? 0ull : ~0ull;
    bool exact = false;                             // wave-uniform

    for (int64_t i0 = 0; i0 < max_len; i0 += STEP) {
        unsigned wv[REGS], won[REGS];
#pragma unroll
        for (int r = 0; r < REGS; ++r) {
            const int64_t i = i0 + r * GW + q;
            wv[r] = (i < len) ? chunk_w[beg + i] : 0u;   // past the end: weight 0 changes nothing
            won[r] = 0;
        }
        if (!exact) {
            unsigned big = 0;
#pragma unroll
            for (int r = 0; r < REGS; ++r) big |= (wv[r] > W_LIMIT) ? 1u : 0u;
            if (__ballot(big != 0) != 0ull) {       // leave the packed representation for good
                exact = true;
                if (has_rail) load = base + (unsigned long long)(key >> S);
            }
        }
        if (!exact) {
            fast_steps<GW, STEP, 0>(key, wv, won, q);
            // advance the base to the current minimum so deltas stay below the packing limit
            const unsigned m = group_min_u32<GW>(key);
            const unsigned adv = (m >> S);
            if (has_rail) { key -= adv << S; base += adv; }
#pragma unroll
            for (int r = 0; r < REGS; ++r) won[r] &= (unsigned)(GW - 1);
        } else {
            exact_steps<GW, STEP, 0>(load, wv, won, q);
        }
#pragma unroll
        for (int r = 0; r < REGS; ++r) {
            const int64_t i = i0 + r * GW + q;
            if (i < len) rail[beg + i] = (uint8_t)won[r];
        }
    }
    if (has_rail) S_out[(int64_t)inst * N + q] = (int64_t)(exact ? load : base + (unsigned long long)(key >> S));
}

template <int GW>
static int launch_lpt(const int64_t *chunk_off, const uint32_t *chunk_w, int64_t n_inst, int N, uint8_t *rail,
                      int64_t *S, hipStream_t st)
{
    constexpr int IPW = 64 / GW;
    const int64_t waves = (n_inst + IPW - 1) / IPW;
    const int64_t blocks = (waves + kLptWaves - 1) / kLptWaves;
    hipLaunchKernelGGL((lpt_spray_kernel<GW>), dim3((unsigned)blocks), dim3(64 * kLptWaves), 0, st, chunk_off, chunk_w,
                       (int)n_inst, N, rail, S);
    return launch_status();
}

}  // namespace rs

extern "C" int railsched_lpt_spray(const int64_t *chunk_off, const uint32_t *chunk_w, int32_t batch,
                                   const railsched_topo_t *h_topo, uint8_t *rail, int64_t *S, void *stream)
{
    using namespace rs;
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0) return RAILSCHED_ERR_INVALID_ARG;
    const int64_t n_inst = (int64_t)batch * h_topo->nodes;
    if (n_inst > 0x7FFFFFFFll / 64) return RAILSCHED_ERR_UNSUPPORTED;
    if (n_inst == 0) return RAILSCHED_OK;
    if (!chunk_off || !S) return RAILSCHED_ERR_NULL_PTR;   // chunk_w / rail may be NULL only when there are no chunks
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int N = h_topo->rails;
    if (N <= 4) return launch_lpt<4>(chunk_off, chunk_w, n_inst, N, rail, S, st);
    if (N <= 8) return launch_lpt<8>(chunk_off, chunk_w, n_inst, N, rail, S, st);
    if (N <= 16) return launch_lpt<16>(chunk_off, chunk_w, n_inst, N, rail, S, st);
    if (N <= 32) return launch_lpt<32>(chunk_off, chunk_w, n_inst, N, rail, S, st);
    return launch_lpt<64>(chunk_off, chunk_w, n_inst, N, rail, S, st);
}
