// Stage 2: GPU-to-GPU traffic matrix D^(1) (Section 4.1; Algorithm 1 step 2).
//
// One workgroup owns (a slice of) the tokens of one (matrix b, source GPU s) pair.  It streams the
// pair's top-k indices with 16-byte loads, maps every (token, slot) to its destination GPU through
// the expert placement table (staged in LDS) and counts hits in an LDS histogram private to the
// workgroup: G 32-bit bins.  Counts become bytes (count * payload) only when the histogram is
// flushed.  HBM traffic is the index stream once plus 8*G bytes per (b, s) pair.
//
// Short-lived workgroups stream best on this chip, so a pair's slots are cut into slices of a few thousand;
// a slice leaves its G counts in the workspace with plain stores and the small reduction kernel shared with
// the one-pass call sums a pair's slices and scales by the payload: no atomics outside LDS, nothing to zero.
#include "common.h"
#include "count_reduce.h"

namespace rs {

constexpr int kTmThreads = 256;    // a slice's workgroup
constexpr int kTmThreadsWhole = 1024;   // the workgroup that takes a whole (matrix, source GPU) pair
constexpr int kTmTableMax = 8192;   // placement entries staged in LDS (32 KiB)

struct TmArgs {
    const int32_t *topk_idx;
    const int32_t *expert_gpu;
    int64_t *D1;
    uint32_t *partial;       // [pairs][splits][G] counts when a pair has several slices
    int64_t slots_per_gpu;   // tokens_per_gpu * k
    int64_t payload;
    int32_t k, kshift;       // kshift >= 0 when k is a power of two
    int32_t E, R, rmask;     // rmask >= 0 when R is a power of two
    int32_t G, splits;
    int32_t copies, lanes_per_period;
    int32_t bin_stride;      // words between histogram copies: odd, so that a bin's copies lie in different LDS banks
    int32_t table_in_lds;
};

template <bool FAST>
__device__ __forceinline__ void tm_count(const TmArgs &a, const int32_t *table, unsigned *bins, int64_t slot, int32_t e)   // bins: this lane's replica
{
    // FAST: k and R are powers of two (shift and mask instead of division)
    const int64_t t = FAST ? (slot >> a.kshift) : (slot / a.k);
    const int rho = FAST ? (int)(t & a.rmask) : (int)(t % a.R);
    if ((unsigned)e < (unsigned)a.E) {
        const int32_t d = table[e * a.R + rho];
        if ((unsigned)d < (unsigned)a.G) atomicAdd(&bins[d], 1u);
    }
}

constexpr int kTmUnroll = 4;        // 16-byte index loads in flight per thread

template <bool FAST, bool TABLE_LDS, int THREADS>
__global__ __launch_bounds__(THREADS) void traffic_matrix_kernel(TmArgs a)
{
    extern __shared__ unsigned tm_lds[];
    // [copies][G] counters.  Lanes whose tokens share a replica index rho - every lanes_per_period-th
    // lane - would pile onto the bins of the popular experts; they get different copies instead.
    unsigned *all_bins = tm_lds;
    unsigned *bins = all_bins + (size_t)((threadIdx.x / a.lanes_per_period) & (a.copies - 1)) * a.bin_stride;
    int32_t *lds_table = reinterpret_cast<int32_t *>(tm_lds + (size_t)a.copies * a.bin_stride);   // [E*R] when it fits
    const int64_t pair = blockIdx.x / a.splits;                         // b*G + s
    const int part = blockIdx.x % a.splits;

    // this workgroup's slice of the pair's slots, cut at multiples of 4 slots
    const int64_t quads = (a.slots_per_gpu + 3) / 4;
    const int64_t qlo = quads * part / a.splits, qhi = quads * (part + 1) / a.splits;
    const int32_t *src = a.topk_idx + pair * a.slots_per_gpu;
    const bool aligned = (reinterpret_cast<uintptr_t>(src) % 16) == 0;
    const int64_t qfull = aligned ? (a.slots_per_gpu / 4 < qhi ? a.slots_per_gpu / 4 : qhi) : qlo;   // whole, aligned quads
    constexpr int64_t kStep = (int64_t)kTmUnroll * THREADS;
    auto whole_step = [&](int64_t q) { return q + (int64_t)(kTmUnroll - 1) * THREADS < qfull; };
    auto request = [&](int64_t q, int4 (&e)[kTmUnroll]) {
#pragma unroll
        for (int u = 0; u < kTmUnroll; ++u) e[u] = *reinterpret_cast<const int4 *>(src + (q + (int64_t)u * THREADS) * 4);
    };
    // the first step's indices are requested before the histogram is cleared and the table staged, every later step's
    // before the step in hand is counted: the loads of a short-lived workgroup are in flight from its first instruction on
    int64_t qd = qlo + threadIdx.x;
    int4 cur[kTmUnroll];
    bool have = whole_step(qd);
    if (have) request(qd, cur);

    for (int i = threadIdx.x; i < a.bin_stride * a.copies; i += THREADS) all_bins[i] = 0;
    if (TABLE_LDS)
        for (int i = threadIdx.x; i < a.E * a.R; i += THREADS) lds_table[i] = a.expert_gpu[i];
    __syncthreads();
    // one definite kind of memory per instantiation: through a pointer that may be LDS or global every lookup is a
    // flat load, which waits for all of the wavefront's memory traffic
    const int32_t *table;
    if constexpr (TABLE_LDS) table = lds_table; else table = a.expert_gpu;

    while (have) {
        int4 nxt[kTmUnroll];
        const bool more = whole_step(qd + kStep);
        if (more) request(qd + kStep, nxt);
#pragma unroll
        for (int u = 0; u < kTmUnroll; ++u) {
            const int64_t s0 = (qd + (int64_t)u * THREADS) * 4;
            tm_count<FAST>(a, table, bins, s0 + 0, cur[u].x);
            tm_count<FAST>(a, table, bins, s0 + 1, cur[u].y);
            tm_count<FAST>(a, table, bins, s0 + 2, cur[u].z);
            tm_count<FAST>(a, table, bins, s0 + 3, cur[u].w);
        }
        qd += kStep;
        have = more;
        if (more) {
#pragma unroll
            for (int u = 0; u < kTmUnroll; ++u) cur[u] = nxt[u];
        }
    }
    for (; qd < qhi; qd += THREADS) {
        const int64_t s0 = qd * 4;
        for (int j = 0; j < 4; ++j)
            if (s0 + j < a.slots_per_gpu) tm_count<FAST>(a, table, bins, s0 + j, src[s0 + j]);
    }
    __syncthreads();

    int64_t *dst = a.D1 + pair * a.G;
    for (int i = threadIdx.x; i < a.G; i += THREADS) {
        unsigned cnt = 0;
        for (int c = 0; c < a.copies; ++c) cnt += all_bins[(size_t)c * a.bin_stride + i];
        if (a.splits == 1) dst[i] = (int64_t)cnt * a.payload;           // sole owner of the pair
        else a.partial[((int64_t)pair * a.splits + part) * a.G + i] = cnt;
    }
}

}  // namespace rs

namespace rs {
// slices per pair: a few thousand slots each, more for large G so that a slice's G counts stay a small share of
// its index bytes
static int64_t tm_splits(int64_t slots_per_gpu, int64_t G, int64_t pairs)
{
    // Enough pairs to fill the chip twice over and few enough slots each: one workgroup of 1024 threads takes the whole pair
    // and writes its D1 row itself - no slice counts, no second kernel (a DeepSeek-V3-shaped layer: 512 pairs of 65 536 slots,
    // 0.038 -> 0.03 ms).
    if (pairs >= 512 && slots_per_gpu <= (int64_t)kTmThreadsWhole * 4 * 32) return 1;
    const int64_t unit = (int64_t)kTmThreads * kTmUnroll * 4;            // slots one workgroup covers per step
    int64_t slice = unit;
    while (slice < 32 * G) slice += unit;
    int64_t splits = (slots_per_gpu + slice - 1) / slice;
    if (splits < 1) splits = 1;
    while (splits > 1 && pairs * splits > 0x7FFFFFFFll) splits = (splits + 1) / 2;
    return splits;
}
}  // namespace rs

extern "C" size_t railsched_traffic_matrix_workspace_bytes(int32_t batch, int64_t tokens_per_gpu, int32_t k,
                                                           const railsched_topo_t *h_topo)
{
    using namespace rs;
    if (check_topo(h_topo) != RAILSCHED_OK || batch < 0 || tokens_per_gpu < 0 || k < 1) return 0;
    const int64_t G = (int64_t)h_topo->nodes * h_topo->rails;
    const int64_t pairs = (int64_t)batch * G;
    if (pairs == 0 || tokens_per_gpu > (int64_t(1) << 31) / k) return 256;
    const int64_t splits = tm_splits(tokens_per_gpu * k, G, pairs);
    return splits > 1 ? align_up(sizeof(uint32_t) * (size_t)(pairs * splits * G), 256) : 256;
}

extern "C" int railsched_traffic_matrix(const int32_t *topk_idx, int32_t batch, int64_t tokens_per_gpu, int32_t k,
                                        const int32_t *expert_gpu, int32_t E, int32_t R, int64_t payload_bytes,
                                        const railsched_topo_t *h_topo, int64_t *D1, void *ws, size_t ws_bytes, void *stream)
{
    using namespace rs;
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0 || tokens_per_gpu < 0 || k < 1 || E < 1 || R < 1 || payload_bytes < 0) return RAILSCHED_ERR_INVALID_ARG;
    if (E > kMaxExperts) return RAILSCHED_ERR_UNSUPPORTED;
    const int64_t G = (int64_t)h_topo->nodes * h_topo->rails;
    if (tokens_per_gpu > (int64_t(1) << 31) / k) return RAILSCHED_ERR_UNSUPPORTED;   // 32-bit bin counters
    if (batch == 0) return RAILSCHED_OK;
    if (!D1 || !expert_gpu || (!topk_idx && tokens_per_gpu > 0)) return RAILSCHED_ERR_NULL_PTR;
    hipStream_t st = static_cast<hipStream_t>(stream);

    TmArgs a;
    a.topk_idx = topk_idx; a.expert_gpu = expert_gpu; a.D1 = D1;
    a.slots_per_gpu = tokens_per_gpu * k; a.payload = payload_bytes;
    a.k = k; a.kshift = is_pow2(k) ? ilog2(k) : -1;
    a.E = E; a.R = R; a.rmask = is_pow2(R) ? R - 1 : -1;
    a.G = (int32_t)G;
    const int64_t pairs = (int64_t)batch * G;
    const int64_t splits = tm_splits(a.slots_per_gpu, G, pairs);
    if (pairs * splits > 0x7FFFFFFFll) return RAILSCHED_ERR_UNSUPPORTED;
    const bool whole = splits == 1 && pairs >= 512 && a.slots_per_gpu > (int64_t)kTmThreads * 4;   // see tm_splits
    a.copies = 1;
    // as many copies as keep a workgroup's LDS (bins + table) within 20 KiB: eight workgroups of 256, all the wavefronts a CU
    // takes (two workgroups of 1024 have 80 KiB each, which the 8192-word bound keeps them far from)
    const int64_t table_words = (int64_t)E * R <= kTmTableMax ? (int64_t)E * R : 0;     // a larger table stays in global memory
    while (a.copies < 8 && (int64_t)a.copies * 2 * (G | 1) <= 8192 &&
           (whole || 4 * ((int64_t)a.copies * 2 * (G | 1) + table_words) <= 20 * 1024))
        a.copies *= 2;
    // a lane holds 4 consecutive slots, so rho repeats every R*k/4 lanes when that is a whole number
    a.lanes_per_period = ((int64_t)R * k % 4 == 0 && (int64_t)R * k / 4 <= 64) ? (int32_t)((int64_t)R * k / 4) : 1;
    a.bin_stride = (int32_t)(a.copies > 1 ? (G | 1) : G);
    a.table_in_lds = ((int64_t)E * R <= kTmTableMax && 4 * (a.copies * (int64_t)a.bin_stride + (int64_t)E * R) <= 64 * 1024) ? 1 : 0;

    a.splits = (int32_t)splits;
    a.partial = static_cast<uint32_t *>(ws);
    if (splits > 1) {
        const size_t need = sizeof(uint32_t) * (size_t)(pairs * splits * G);
        if (!ws || ws_bytes < need || reinterpret_cast<uintptr_t>(ws) % 4 != 0) return RAILSCHED_ERR_WORKSPACE;
    }
    const size_t lds = sizeof(unsigned) * (size_t)a.bin_stride * a.copies + (a.table_in_lds ? sizeof(int32_t) * (size_t)E * R : 0);
    const dim3 grid((unsigned)(pairs * splits));
    const bool fast = a.kshift >= 0 && a.rmask >= 0;
    if (whole) {
        constexpr int T = kTmThreadsWhole;
        if (fast && a.table_in_lds) hipLaunchKernelGGL((traffic_matrix_kernel<true, true, T>), grid, dim3(T), lds, st, a);
        else if (fast) hipLaunchKernelGGL((traffic_matrix_kernel<true, false, T>), grid, dim3(T), lds, st, a);
        else if (a.table_in_lds) hipLaunchKernelGGL((traffic_matrix_kernel<false, true, T>), grid, dim3(T), lds, st, a);
        else hipLaunchKernelGGL((traffic_matrix_kernel<false, false, T>), grid, dim3(T), lds, st, a);
    } else {
        constexpr int T = kTmThreads;
        if (fast && a.table_in_lds) hipLaunchKernelGGL((traffic_matrix_kernel<true, true, T>), grid, dim3(T), lds, st, a);
        else if (fast) hipLaunchKernelGGL((traffic_matrix_kernel<true, false, T>), grid, dim3(T), lds, st, a);
        else if (a.table_in_lds) hipLaunchKernelGGL((traffic_matrix_kernel<false, true, T>), grid, dim3(T), lds, st, a);
        else hipLaunchKernelGGL((traffic_matrix_kernel<false, false, T>), grid, dim3(T), lds, st, a);
    }
    if (int rc = launch_status()) return rc;
    if (splits > 1) return launch_count_reduce(a.partial, D1, pairs * G, (int)G, (int)splits, payload_bytes, st);
    return RAILSCHED_OK;
}
