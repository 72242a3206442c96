// Stages 1 and 2 in one pass (Algorithm 1 steps 1-2): the gating decision of every token and the
// GPU-to-GPU traffic matrix D^(1) it implies, without reading the indices back from memory.
//
// For rows of at most 8 logits a lane holds a whole row, so the lane that picks a row's k experts
// also knows the row's source GPU and replica index: it bumps the destination's bin in an LDS
// histogram of the workgroup (which owns a slice of one (matrix, source GPU) pair's tokens) right
// after the pick.  HBM traffic is the logits once, plus the indices once if the caller wants them;
// the separate stage 2 would read them again.  The picks are made by the same comparisons as stage 1
// (strict '>' in ascending expert index, winners replaced by -inf), so both outputs are bit-identical
// to the two separate calls.
// Rows of 33..256 logits with k <= 8 have a one-pass kernel too, for callers that do not want the indices: the
// insertion kernel of stage 1 with the same addition - once the lanes of a row hold its winners, lane j looks up
// the destination of winner j and bumps its bin.  A workgroup walks a few hundred consecutive tokens of one pair
// so that its G counts are a small share of the logits it read.  When the indices are wanted the two stages run
// back to back instead: measured on 4 194 304 rows of 256 logits, top-8, the one-pass kernel takes 0.74 ms without
// and 0.80 ms with the index stores (its workgroups live eight times longer than stage 1's, which ends the launch
// on a longer tail), the two separate kernels 0.72 + 0.04 ms.  Other shapes always run the two stages.
//
// Short-lived workgroups of one or a few rounds of 512 tokens stream best, so a pair's tokens are cut
// into many slices; each slice leaves its G counts in the workspace with plain stores and a second,
// small kernel sums a pair's slices and scales by the payload.
#include "common.h"
#include "count_reduce.h"
#include "topk_core.h"

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

// ---------------------------------------------------------------------------------------------- rows of 33..256 logits
struct RwArgs {
    const float *logits;
    const int32_t *expert_gpu;
    int64_t *D1;
    uint32_t *partial;       // [pairs][splits][G] counts when a pair has several slices
    int64_t tokens_per_gpu;
    int64_t payload;
    int32_t E, k, R, rmask;  // rmask >= 0 when R is a power of two
    int32_t G, splits;
    int32_t iters;           // row groups (of 4 * 64/LANES tokens) a workgroup walks
    int32_t table_in_lds;
};

template <int LANES, int VPL, int L, int WAVES, bool FULL, bool TABLE_LDS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WAVES, 8))) void route_traffic_insert_kernel(RwArgs a)
{
    extern __shared__ unsigned rw_lds[];
    constexpr int RPW = 64 / LANES;                 // rows per wavefront
    constexpr int RPB = 4 * RPW;                    // rows per workgroup and iteration
    constexpr unsigned MASK = (unsigned)(LANES * VPL) - 1u;
    unsigned *bins = rw_lds;                        // [G] destination counts of this workgroup's tokens
    int32_t *lds_table = reinterpret_cast<int32_t *>(rw_lds + a.G);
    const int64_t pair = blockIdx.x / a.splits;     // b*G + s
    const int part = blockIdx.x % a.splits;
    const int lane = threadIdx.x & 63;
    const int q = lane % LANES;

    for (int i = threadIdx.x; i < a.G; i += 256) bins[i] = 0;
    if (TABLE_LDS)
        for (int i = threadIdx.x; i < a.E * a.R; i += 256) lds_table[i] = a.expert_gpu[i];
    __syncthreads();
    const int32_t *table;
    if constexpr (TABLE_LDS) table = lds_table; else table = a.expert_gpu;   // one definite kind of memory per instantiation

    const int64_t t_lo = (int64_t)part * a.iters * RPB;
    const float *pair_logits = a.logits + pair * a.tokens_per_gpu * a.E;
    const int64_t t_first = t_lo + (threadIdx.x >> 6) * RPW + lane / LANES;     // this lane's token in the first row group
    auto clamp_token = [&](int64_t t) { return t < a.tokens_per_gpu ? t : a.tokens_per_gpu - 1; };
    float4 x[VPL / 4];
    row_load<LANES, VPL, FULL>(pair_logits + clamp_token(t_first) * a.E, a.E, q, x);
    for (int it = 0; it < a.iters; ++it) {
        if (t_lo + (int64_t)it * RPB >= a.tokens_per_gpu) break;                 // workgroup-uniform
        const int64_t t = t_first + (int64_t)it * RPB;                           // token inside the pair
        const bool live = t < a.tokens_per_gpu;
        const int rho = a.rmask >= 0 ? (int)(t & a.rmask) : (int)(t % a.R);
        auto count = [&](int e) {
            if ((unsigned)e < (unsigned)a.E) {
                const int32_t d = table[e * a.R + rho];
                if ((unsigned)d < (unsigned)a.G) atomicAdd(&bins[d], 1u);
            }
        };
        float own[L];
        lane_best<LANES, VPL, L>(x, q, own);
        // the next row group's logits are requested as soon as this one's are consumed
        if (it + 1 < a.iters) row_load<LANES, VPL, FULL>(pair_logits + clamp_token(t + RPB) * a.E, a.E, q, x);
        unsigned u[8];
        const bool bad = row_best8<LANES, VPL, L>(own, a.k, u);
        if (__ballot(live && bad) == 0ull) {
#pragma unroll
            for (int r = 0; r < (8 + LANES - 1) / LANES; ++r) {          // winners q, q+LANES, ... are counted by this lane
                unsigned sel = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) sel = (j == q + r * LANES) ? u[j] : sel;
                if (live && q + r * LANES < a.k) count((int)(sel & MASK));
            }
        } else {
            // rare: the wavefront's rows are read again and picked by full comparisons
            row_exact<LANES, VPL>(pair_logits + t * a.E, live, a.E, a.k, q, [&](int sel, int bi) {
                if (live && q == sel % LANES) count(bi);
            });
        }
    }
    __syncthreads();
    int64_t *dst = a.D1 + pair * a.G;
    for (int i = threadIdx.x; i < a.G; i += 256) {
        if (a.splits == 1) dst[i] = (int64_t)bins[i] * a.payload;      // sole owner of the pair
        else a.partial[((int64_t)pair * a.splits + part) * a.G + i] = bins[i];
    }
}

// row groups per workgroup: enough tokens that the G counts a workgroup leaves behind are under a hundredth of the logits it read
static int rw_iters(int64_t tokens_per_gpu, int64_t G, int E, int rows_per_group)
{
    int64_t it = 1;
    while (it * rows_per_group * E < 128 * G && it * rows_per_group < tokens_per_gpu) it *= 2;
    return (int)it;
}

template <int LANES, int VPL, int L, int WAVES>
static int launch_route_traffic_insert(RwArgs a, int64_t pairs, hipStream_t st)
{
    const size_t lds = sizeof(unsigned) * (size_t)a.G + (a.table_in_lds ? sizeof(int32_t) * (size_t)a.E * a.R : 0);
    const dim3 grid((unsigned)(pairs * a.splits));
    const bool full = a.E == LANES * VPL;
#define RW_LAUNCH(FULL_, TAB_) hipLaunchKernelGGL((route_traffic_insert_kernel<LANES, VPL, L, WAVES, FULL_, TAB_>), grid, dim3(256), lds, st, a)
    if (full && a.table_in_lds) RW_LAUNCH(true, true);
    else if (full) RW_LAUNCH(true, false);
    else if (a.table_in_lds) RW_LAUNCH(false, true);
    else RW_LAUNCH(false, false);
#undef RW_LAUNCH
    return launch_status();
}

// shape of the one-pass kernel for rows of 33..256 logits; false: the two stages run back to back
static bool rw_shape(const float *logits, int32_t E, int32_t k, int64_t G, int *lanes)
{
    const bool vec4 = (E % 4 == 0) && (reinterpret_cast<uintptr_t>(logits) % 16 == 0);
    if (!vec4 || E <= 32 || E > 256 || k > 8) return false;
    if (4 * G > 16 * 1024) return false;            // the destination counts of a workgroup live in LDS
    *lanes = E <= 128 ? 4 : 8;
    return true;
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
    if (E > 8) {
        // the larger of what the one-pass kernel for 33..256 logits and the two-stage path would need
        size_t need = railsched_traffic_matrix_workspace_bytes(batch, tokens_per_gpu, k, h_topo);
        const int rpg = 4 * (64 / (E <= 128 ? 4 : 8));
        if (E > 32 && E <= 256 && k <= 8 && pairs > 0 && 4 * G <= 16 * 1024) {
            const int64_t rb = (int64_t)rw_iters(tokens_per_gpu, G, E, rpg) * rpg;
            const int64_t splits = (tokens_per_gpu + rb - 1) / rb;
            const size_t one = splits > 1 ? align_up(sizeof(uint32_t) * (size_t)(pairs * splits * G), 256) : 256;
            need = one > need ? one : need;
        }
        return need;
    }
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

    int lanes = 0;
    if (E > 8 && rows > 0 && !topk_idx && rw_shape(logits, E, k, G, &lanes)) {
        // the indices are not wanted: one pass (with them, the two stages below are the faster way on this chip)
        RwArgs a;
        a.logits = logits; a.expert_gpu = expert_gpu; a.D1 = D1;
        a.tokens_per_gpu = tokens_per_gpu; a.payload = payload_bytes;
        a.E = E; a.k = k; a.R = R; a.rmask = is_pow2(R) ? R - 1 : -1;
        a.G = (int32_t)G;
        const int rpg = 4 * (64 / lanes);
        a.iters = rw_iters(tokens_per_gpu, G, E, rpg);
        const int64_t rb = (int64_t)a.iters * rpg;
        const int64_t splits = (tokens_per_gpu + rb - 1) / rb;
        if (pairs * splits > 0x7FFFFFFFll) return RAILSCHED_ERR_UNSUPPORTED;
        a.splits = (int32_t)splits;
        a.partial = static_cast<uint32_t *>(ws);
        if (splits > 1) {
            const size_t need = sizeof(uint32_t) * (size_t)(pairs * splits * G);
            if (!ws || ws_bytes < need || reinterpret_cast<uintptr_t>(ws) % 4 != 0) return RAILSCHED_ERR_WORKSPACE;
        }
        a.table_in_lds = ((int64_t)E * R <= kRtTableMax && 4 * (G + (int64_t)E * R) <= 16 * 1024) ? 1 : 0;
        hipStream_t st = static_cast<hipStream_t>(stream);
        int rc;
        if (E <= 64) rc = launch_route_traffic_insert<4, 16, 8, 6>(a, pairs, st);
        else if (E <= 128) rc = launch_route_traffic_insert<4, 32, 8, 4>(a, pairs, st);
        else rc = launch_route_traffic_insert<8, 32, 6, 4>(a, pairs, st);
        if (rc) return rc;
        if (splits > 1) return launch_count_reduce(a.partial, D1, pairs * G, (int)G, (int)splits, payload_bytes, st);
        return RAILSCHED_OK;
    }
    if (E > 8) {
        // other shapes: the two stages run one after the other through the index array
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
