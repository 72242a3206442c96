// Stages 1 and 2 in one pass (Algorithm 1 steps 1-2): the gating decision of every token and the
// GPU-to-GPU traffic matrix D^(1) it implies, without reading the indices back from memory.
//
// For rows of at most 8 logits a lane holds a whole row, so the lane that picks a row's k experts
// also knows the row's source GPU and replica index: it bumps the destination's bin in an LDS
// histogram of the workgroup (which owns a slice of one (matrix, source GPU) pair's tokens) right
// after the pick.  HBM traffic is the logits once, plus the indices once if the caller wants them;
// the separate stage 2 would read them again.  The picks are made by the same comparisons as stage 1
// (strict '>' in ascending expert index, winners replaced by -inf), so both outputs are bit-identical
// to the two separate calls.  Wider rows run the two stages back to back.
//
// Short-lived workgroups of one or a few rounds of 512 tokens stream best, so a pair's tokens are cut
// into many slices; each slice leaves its G counts in the workspace with plain stores and a second,
// small kernel sums a pair's slices and scales by the payload.
#include "common.h"
#include "count_reduce.h"

#include <cfloat>
#include <climits>

namespace rs {

typedef float rt_f32x4 __attribute__((ext_vector_type(4)));
typedef int rt_i32x2 __attribute__((ext_vector_type(2)));

constexpr int kRtThreads = 256;
constexpr int kRtUnroll = 2;          // rows per thread with their loads in flight together
constexpr int kRtRound = kRtThreads * kRtUnroll;   // tokens per workgroup and round
constexpr int kRtTableMax = 8192;     // placement entries staged in LDS

struct RtArgs {
    const float *logits;
    const int32_t *expert_gpu;
    int32_t *topk_idx;       // may be null: the picks are only counted
    int64_t *D1;
    uint32_t *partial;       // [pairs][splits][G] counts when a pair has several slices
    int64_t tokens_per_gpu;
    int64_t payload;
    int32_t E, k, R, rmask;  // rmask >= 0 when R is a power of two
    int32_t G, splits;
    int32_t copies, lanes_per_period;
    int32_t bin_stride;      // words between histogram copies: odd, so that a bin's copies lie in different LDS banks
    int32_t table_in_lds;
};

// D1[pair][d] = payload * sum of the pair's slice counts
__global__ __launch_bounds__(256) void rt_reduce_kernel(const uint32_t *__restrict__ partial, int64_t *__restrict__ D1, int64_t n, int G,
                                                        int splits, int64_t payload)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t pair = i / G;
        const int d = (int)(i - pair * G);
        const uint32_t *src = partial + pair * splits * G + d;
        uint64_t cnt = 0;
        int p = 0;
        for (; p + 8 <= splits; p += 8) {                    // eight independent loads in flight
            uint32_t x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = src[(int64_t)(p + u) * G];
#pragma unroll
            for (int u = 0; u < 8; ++u) cnt += x[u];
        }
        for (; p < splits; ++p) cnt += src[(int64_t)p * G];
        D1[i] = (int64_t)cnt * payload;
    }
}

int launch_count_reduce(const uint32_t *partial, int64_t *D1, int64_t n, int G, int splits, int64_t payload, hipStream_t st)
{
    const int64_t blocks = (n + 255) / 256 > 65536 ? 65536 : (n + 255) / 256;
    hipLaunchKernelGGL(rt_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st, partial, D1, n, G, splits, payload);
    return launch_status();
}

template <int VPL, bool VEC4>
__device__ __forceinline__ void rt_load_row(const RtArgs &a, int64_t row, bool live, float (&v)[VPL])
{
    if constexpr (VEC4) {
#pragma unroll
        for (int c = 0; c < VPL / 4; ++c) {
            rt_f32x4 x = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            if (live && 4 * c < a.E) x = __builtin_nontemporal_load(reinterpret_cast<const rt_f32x4 *>(a.logits + row * a.E + 4 * c));
            v[4 * c + 0] = x.x; v[4 * c + 1] = x.y; v[4 * c + 2] = x.z; v[4 * c + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < VPL; ++j) v[j] = (live && j < a.E) ? a.logits[row * a.E + j] : -INFINITY;
    }
}

// picks of one row, largest first, lowest index on ties; counts each pick's destination GPU.  With k = 2 the two
// winners come back in `pair` and the caller stores them once all its rows are picked: a store between two rows
// made the second row's table lookups wait for it (memory operations of a wavefront complete in order).
template <int VPL>
__device__ __forceinline__ void rt_pick_row(const RtArgs &a, const int32_t *table, unsigned *bins, int64_t row, int64_t t_local,
                                            float (&v)[VPL], rt_i32x2 &pair)
{
    const int rho = a.rmask >= 0 ? (int)(t_local & a.rmask) : (int)(t_local % a.R);
    int keep0 = 0;
    for (int sel = 0; sel < a.k; ++sel) {
        float bv = -INFINITY;
        int bi = INT_MAX;
#pragma unroll
        for (int j = 0; j < VPL; ++j) {
            const bool better = v[j] > bv;
            bv = better ? v[j] : bv;
            bi = better ? j : bi;
        }
#pragma unroll
        for (int j = 0; j < VPL; ++j) v[j] = (j == bi) ? -INFINITY : v[j];
        if ((unsigned)bi < (unsigned)a.E) {
            const int32_t d = table[bi * a.R + rho];
            if ((unsigned)d < (unsigned)a.G) atomicAdd(&bins[d], 1u);
        }
        if (a.k == 2) {                                       // both winners leave in one 8-byte store, issued by the caller
            if (sel == 0) keep0 = bi;
            else { pair.x = keep0; pair.y = bi; }
        } else if (a.topk_idx) {
            a.topk_idx[row * a.k + sel] = bi;
        }
    }
}

template <int VPL, bool VEC4, bool TABLE_LDS>
__global__ __launch_bounds__(kRtThreads) void route_traffic_kernel(RtArgs a)
{
    extern __shared__ unsigned rt_lds[];
    // [copies][G] counters; lanes that share a replica index - every lanes_per_period-th lane - would pile
    // onto the bins of the popular experts, so neighbouring periods count in different copies
    unsigned *all_bins = rt_lds;
    unsigned *bins = all_bins + (size_t)((threadIdx.x / a.lanes_per_period) & (a.copies - 1)) * a.bin_stride;
    int32_t *lds_table = reinterpret_cast<int32_t *>(rt_lds + (size_t)a.copies * a.bin_stride);
    const int64_t pair = blockIdx.x / a.splits;              // b*G + s
    const int part = blockIdx.x % a.splits;

    // the pair's tokens are dealt to its workgroups in rounds of kRtRound, so the workgroups of a
    // pair, which are dispatched together, sweep one contiguous window of the logits side by side
    const int64_t hi = a.tokens_per_gpu;
    const int64_t row0 = pair * a.tokens_per_gpu;
    const int64_t round = (int64_t)a.splits * kRtRound;
    int64_t t = (int64_t)part * kRtRound + threadIdx.x;
    float v[kRtUnroll][VPL];
    // the first round's logits are requested before the histogram is set up, so that clearing it and
    // fetching the placement table do not delay them
#pragma unroll
    for (int u = 0; u < kRtUnroll; ++u) {
        const int64_t tu = t + (int64_t)u * kRtThreads;
        rt_load_row<VPL, VEC4>(a, row0 + tu, tu < hi, v[u]);
    }

    for (int i = threadIdx.x; i < a.bin_stride * a.copies; i += kRtThreads) all_bins[i] = 0;
    if (TABLE_LDS)
        for (int i = threadIdx.x; i < a.E * a.R; i += kRtThreads) lds_table[i] = a.expert_gpu[i];
    __syncthreads();

    while (t < hi) {
        rt_i32x2 pairs[kRtUnroll];
#pragma unroll
        for (int u = 0; u < kRtUnroll; ++u) {
            const int64_t tu = t + (int64_t)u * kRtThreads;
            pairs[u].x = 0; pairs[u].y = 0;
            // two calls, so that the table is read with LDS instructions where it is in LDS: through one pointer
            // that may be either, every lookup waited for all of the wavefront's memory traffic
            if (tu < hi) {
                if (TABLE_LDS) rt_pick_row<VPL>(a, lds_table, bins, row0 + tu, tu, v[u], pairs[u]);
                else rt_pick_row<VPL>(a, a.expert_gpu, bins, row0 + tu, tu, v[u], pairs[u]);
            }
        }
        if (a.topk_idx && a.k == 2) {
#pragma unroll
            for (int u = 0; u < kRtUnroll; ++u) {
                const int64_t tu = t + (int64_t)u * kRtThreads;
                if (tu < hi) __builtin_nontemporal_store(pairs[u], reinterpret_cast<rt_i32x2 *>(a.topk_idx + (row0 + tu) * 2));
            }
        }
        t += round;
        if (t >= hi) break;
#pragma unroll
        for (int u = 0; u < kRtUnroll; ++u) {
            const int64_t tu = t + (int64_t)u * kRtThreads;
            rt_load_row<VPL, VEC4>(a, row0 + tu, tu < hi, v[u]);
        }
    }
    __syncthreads();

    int64_t *dst = a.D1 + pair * a.G;
    for (int i = threadIdx.x; i < a.G; i += kRtThreads) {
        unsigned cnt = 0;
        for (int c = 0; c < a.copies; ++c) cnt += all_bins[(size_t)c * a.bin_stride + i];
        if (a.splits == 1) dst[i] = (int64_t)cnt * a.payload;    // sole owner of the pair
        else a.partial[((int64_t)pair * a.splits + part) * a.G + i] = cnt;
    }
}

template <int VPL>
static int launch_route_traffic(const RtArgs &a, int64_t pairs, size_t lds, hipStream_t st)
{
    const bool vec4 = (a.E % 4 == 0) && (reinterpret_cast<uintptr_t>(a.logits) % 16 == 0);
    const dim3 grid((unsigned)(pairs * a.splits));
    if (vec4 && a.table_in_lds) hipLaunchKernelGGL((route_traffic_kernel<VPL, true, true>), grid, dim3(kRtThreads), lds, st, a);
    else if (vec4) hipLaunchKernelGGL((route_traffic_kernel<VPL, true, false>), grid, dim3(kRtThreads), lds, st, a);
    else if (a.table_in_lds) hipLaunchKernelGGL((route_traffic_kernel<VPL, false, true>), grid, dim3(kRtThreads), lds, st, a);
    else hipLaunchKernelGGL((route_traffic_kernel<VPL, false, false>), grid, dim3(kRtThreads), lds, st, a);
    return launch_status();
}

}  // namespace rs

namespace rs {
// slices per pair: one round of tokens per slice while that keeps the slice counts (4*G bytes per slice)
// a small fraction of the logits, more rounds per slice for large G
static int64_t rt_splits(int64_t tokens_per_gpu, int64_t G, int64_t pairs)
{
    const int64_t rounds = (8 * G + kRtRound - 1) / kRtRound;
    const int64_t slice = kRtRound * (rounds < 1 ? 1 : rounds);
    int64_t splits = (tokens_per_gpu + slice - 1) / slice;
    if (splits < 1) splits = 1;
    while (splits > 1 && pairs * splits > 0x7FFFFFFFll) splits = (splits + 1) / 2;
    return splits;
}
}  // namespace rs

extern "C" size_t railsched_route_traffic_workspace_bytes(int32_t batch, int64_t tokens_per_gpu, int32_t E, int32_t k,
                                                          const railsched_topo_t *h_topo)
{
    using namespace rs;
    if (check_topo(h_topo) != RAILSCHED_OK || batch < 0 || tokens_per_gpu < 0 || E < 1 || k < 1) return 0;
    const int64_t G = (int64_t)h_topo->nodes * h_topo->rails;
    const int64_t pairs = (int64_t)batch * G;
    if (E > 8) return railsched_traffic_matrix_workspace_bytes(batch, tokens_per_gpu, k, h_topo);
    if (pairs == 0) return 256;
    const int64_t splits = rt_splits(tokens_per_gpu, G, pairs);
    return splits > 1 ? align_up(sizeof(uint32_t) * (size_t)(pairs * splits * G), 256) : 256;
}

extern "C" int railsched_route_traffic(const float *logits, int32_t batch, int64_t tokens_per_gpu, int32_t E, int32_t k,
                                       const int32_t *expert_gpu, int32_t R, int64_t payload_bytes,
                                       const railsched_topo_t *h_topo, int32_t *topk_idx, int64_t *D1, void *ws,
                                       size_t ws_bytes, void *stream)
{
    using namespace rs;
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0 || tokens_per_gpu < 0 || E < 1 || k < 1 || k > E || R < 1 || payload_bytes < 0) return RAILSCHED_ERR_INVALID_ARG;
    if (E > kMaxExperts) return RAILSCHED_ERR_UNSUPPORTED;
    const int64_t G = (int64_t)h_topo->nodes * h_topo->rails;
    if (tokens_per_gpu > (int64_t(1) << 31) / k) return RAILSCHED_ERR_UNSUPPORTED;   // 32-bit bin counters
    if (batch == 0) return RAILSCHED_OK;
    if (!D1 || !expert_gpu || (!logits && tokens_per_gpu > 0)) return RAILSCHED_ERR_NULL_PTR;
    const int64_t pairs = (int64_t)batch * G;
    const int64_t rows = pairs * tokens_per_gpu;

    if (E > 8) {
        // a row spans several lanes: the two stages run one after the other through the index array
        if (!topk_idx && rows > 0) return RAILSCHED_ERR_NULL_PTR;
        if (int rc = railsched_route_topk(logits, rows, E, k, topk_idx, stream)) return rc;
        return railsched_traffic_matrix(topk_idx, batch, tokens_per_gpu, k, expert_gpu, E, R, payload_bytes, h_topo, D1, ws, ws_bytes, stream);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);

    RtArgs a;
    a.logits = logits; a.expert_gpu = expert_gpu; a.topk_idx = topk_idx; a.D1 = D1;
    a.tokens_per_gpu = tokens_per_gpu; a.payload = payload_bytes;
    a.E = E; a.k = k; a.R = R; a.rmask = is_pow2(R) ? R - 1 : -1;
    a.G = (int32_t)G;
    a.copies = 1;
    while (a.copies < 8 && (int64_t)a.copies * 2 * (G | 1) <= 8192) a.copies *= 2;
    a.lanes_per_period = R <= 64 ? R : 1;                    // a lane holds one token, so rho repeats every R lanes
    a.bin_stride = (int32_t)(a.copies > 1 ? (G | 1) : G);
    a.table_in_lds = ((int64_t)E * R <= kRtTableMax && 4 * (a.copies * (int64_t)a.bin_stride + (int64_t)E * R) <= 64 * 1024) ? 1 : 0;

    const int64_t splits = rt_splits(tokens_per_gpu, G, pairs);
    if (pairs * splits > 0x7FFFFFFFll) return RAILSCHED_ERR_UNSUPPORTED;
    a.splits = (int32_t)splits;
    a.partial = static_cast<uint32_t *>(ws);
    if (splits > 1) {
        const size_t need = sizeof(uint32_t) * (size_t)(pairs * splits * G);
        if (!ws || ws_bytes < need || reinterpret_cast<uintptr_t>(ws) % 4 != 0) return RAILSCHED_ERR_WORKSPACE;
    }
    const size_t lds = sizeof(unsigned) * (size_t)a.bin_stride * a.copies + (a.table_in_lds ? sizeof(int32_t) * (size_t)E * R : 0);
    if (int rc = E <= 4 ? launch_route_traffic<4>(a, pairs, lds, st) : launch_route_traffic<8>(a, pairs, lds, st)) return rc;
    if (splits > 1) return launch_count_reduce(a.partial, D1, pairs * G, (int)G, (int)splits, payload_bytes, st);
    return RAILSCHED_OK;
}
