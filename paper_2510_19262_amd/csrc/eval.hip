// Stage 5: send/receive loads, completion time and lower bound
// (Section 4.1 load matrices S and R; Theorem 2; Theorem 3; Algorithm 2 step 6 uses the same loads).
//
// Rail n of a source node ends on NIC n of the destination node (one-to-one rail mapping used in the
// proof of Theorem 3), so R[b][f][n] is the sum of the weights of all chunks of matrix b whose
// destination GPU lies in node f and that were assigned to rail n - whatever their source node.
// Kernel 1: the chunk range of matrix b is dealt in rounds to `slices` workgroups; one workgroup streams its
// share (9 bytes per chunk), accumulates the G = M*N receive bins in LDS and writes them, plus the
// largest weight it saw, to its own slot of the workspace with plain stores.
// Kernel 2: one workgroup per matrix adds the slots and derives the statistics from S (as produced by
// stage 4) and R.  No global atomics anywhere; all sums are integer, so their order cannot matter.
#include "common.h"
#include "eval_core.h"

namespace rs {

__global__ __launch_bounds__(kEvThreads) void eval_partial_kernel(EvArgs a)
{
    // [copies][G + 1] 64-bit bins.  Consecutive records mostly go to one destination node and cycle through the
    // rails, so the lanes of a wavefront would pile onto a handful of bins; lanes take different copies instead, and
    // the odd stride puts a bin's copies in different banks.
    extern __shared__ unsigned long long ev_all[];
    __shared__ unsigned ev_wmax;
    if (a.chunk_off[a.n_inst] > a.capacity) return;                     // the record arrays hold nothing
    const int b = blockIdx.y, t = blockIdx.x;
    const int stride = a.G + 1;
    for (int i = threadIdx.x; i < stride * a.copies; i += kEvThreads) ev_all[i] = 0;
    if (threadIdx.x == 0) ev_wmax = 0;
    __syncthreads();
    unsigned long long *ev_bins = ev_all + (size_t)(((threadIdx.x & 63) >> 1) & (a.copies - 1)) * stride;

    // matrix b's records are dealt to its `slices` workgroups in rounds of kEvThreads*4, so the workgroups, which run
    // side by side, read one compact window of the arrays at any time
    const int64_t lo = a.chunk_off[(int64_t)b * a.M], hi = a.chunk_off[(int64_t)(b + 1) * a.M];
    unsigned wmax = 0;
    auto one = [&](uint32_t w, uint32_t flow, unsigned r) {
        const int f = dst_node(a, flow);
        if (f < a.M && r < (unsigned)a.N) atomicAdd(&ev_bins[f * a.N + r], (unsigned long long)w);   // LDS, workgroup-private
        wmax = w > wmax ? w : wmax;
    };
    // whole groups of four records: 16-byte loads of weight and flow, 4 bytes of rails; the first group sits on a
    // 1 KiB boundary of the weight array (256 records), so every wavefront loads whole aligned kilobytes
    const int64_t alo = a.wide_ok ? ((lo + 255) & ~int64_t(255)) : hi, ahi = a.wide_ok ? (hi & ~int64_t(3)) : hi;
    if (alo < ahi) {
        const int64_t round = (int64_t)a.slices * kEvThreads * 4;
        for (int64_t i = alo + ((int64_t)t * kEvThreads + threadIdx.x) * 4; i < ahi; i += round) {
            const uint4 w = *reinterpret_cast<const uint4 *>(a.chunk_w + i);
            const uint4 fl = *reinterpret_cast<const uint4 *>(a.chunk_flow + i);
            const uint32_t rr = *reinterpret_cast<const uint32_t *>(a.rail + i);
            one(w.x, fl.x, rr & 255u); one(w.y, fl.y, (rr >> 8) & 255u); one(w.z, fl.z, (rr >> 16) & 255u); one(w.w, fl.w, rr >> 24);
        }
        const int64_t n_edge = (alo - lo) + (hi - ahi);                 // at most 258 records outside the aligned span
        if (t == 0)
            for (int64_t e = threadIdx.x; e < n_edge; e += kEvThreads) {
                const int64_t i = e < alo - lo ? lo + e : ahi + (e - (alo - lo));
                one(a.chunk_w[i], a.chunk_flow[i], a.rail[i]);
            }
    } else {
        for (int64_t i = lo + (int64_t)t * kEvThreads + threadIdx.x; i < hi; i += (int64_t)a.slices * kEvThreads)
            one(a.chunk_w[i], a.chunk_flow[i], a.rail[i]);
    }
    atomicMax(&ev_wmax, wmax);
    __syncthreads();
    int64_t *slot = a.partial + ((int64_t)b * a.slices + t) * (a.G + 1);
    for (int i = threadIdx.x; i < a.G; i += kEvThreads) {
        unsigned long long sum = 0;
        for (int c = 0; c < a.copies; ++c) sum += ev_all[(size_t)c * stride + i];
        slot[i] = (int64_t)sum;
    }
    if (threadIdx.x == 0) slot[a.G] = (int64_t)ev_wmax;
}

// One workgroup of THREADS/64 wavefronts per matrix (1024 threads, or 256 when the matrix is small: fewer
// wavefronts make cheaper barriers).  Receive bins: a wavefront covers 64 consecutive bins (or, when G < 64,
// several slices side by side), the wavefronts split the slices, LDS joins them.  The six statistics are
// reduced together: shuffles inside the wavefronts, one exchange through LDS.
// R[b][base..base+63] = sum over the matrix's slots, for matrices with so many slots that one workgroup per matrix
// would read megabytes alone: grid (ceil(G/64), batch), four wavefronts split the slots.
__global__ __launch_bounds__(256) void eval_sum_kernel(EvArgs a)
{
    __shared__ int64_t part[4][64];
    if (a.chunk_off[a.n_inst] > a.capacity) return;
    const int b = blockIdx.y, base = blockIdx.x * 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t *slots = a.partial + (int64_t)b * a.slices * (a.G + 1);
    const int i = base + lane;
    int64_t acc = 0;
    if (i < a.G) {
        int t = wave;
        for (; t + 12 < a.slices; t += 16) {              // four independent loads in flight
            const int64_t x0 = slots[(int64_t)t * (a.G + 1) + i], x1 = slots[(int64_t)(t + 4) * (a.G + 1) + i];
            const int64_t x2 = slots[(int64_t)(t + 8) * (a.G + 1) + i], x3 = slots[(int64_t)(t + 12) * (a.G + 1) + i];
            acc += (x0 + x1) + (x2 + x3);
        }
        for (; t < a.slices; t += 4) acc += slots[(int64_t)t * (a.G + 1) + i];
    }
    part[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && i < a.G) a.R[(int64_t)b * a.G + i] = part[0][lane] + part[1][lane] + part[2][lane] + part[3][lane];
}

// SUM: the receive bins are summed here; otherwise eval_sum_kernel has already written R.
template <int THREADS, bool SUM>
__global__ __launch_bounds__(THREADS) void eval_reduce_kernel(EvArgs a)
{
    constexpr int WAVES = THREADS / 64;
    __shared__ int64_t part[WAVES][64];
    __shared__ int64_t sh[6][WAVES];
    const int b = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t *slots = a.partial + (int64_t)b * a.slices * (a.G + 1);
    int64_t *Rb = a.R + (int64_t)b * a.G;
    const int64_t *Sb = a.S + (int64_t)b * a.G;
    if (a.chunk_off[a.n_inst] > a.capacity) {         // more chunks than the record arrays hold: nothing was read, say so
        for (int i = threadIdx.x; i < a.G; i += THREADS) Rb[i] = -1;
        if (threadIdx.x < 8) a.stats[(int64_t)b * 8 + threadIdx.x] = -1;
        return;
    }

    int width = 64;                                   // lanes per slice row: 64, or the power of two >= G
    while (width / 2 >= a.G) width /= 2;
    const int sub = 64 / width;                       // slices a wavefront reads side by side
    const int ts = lane / width, li = lane % width;
    for (int base = 0; SUM && base < a.G; base += 64) {
        const int i = base + li;
        int64_t acc = 0;
        if (i < a.G)
            for (int t = wave * sub + ts; t < a.slices; t += WAVES * sub) acc += slots[(int64_t)t * (a.G + 1) + i];
        __syncthreads();                              // previous round's readers are done
        part[wave][lane] = acc;
        __syncthreads();
        if (wave == 0 && lane < width && base + lane < a.G) {
            int64_t r = 0;
            for (int w = 0; w < WAVES; ++w)
                for (int u = 0; u < sub; ++u) r += part[w][u * width + lane];
            Rb[base + lane] = r;
        }
    }
    int64_t wmax = 0;
    for (int t = threadIdx.x; t < a.slices; t += THREADS) {
        const int64_t x = slots[(int64_t)t * (a.G + 1) + a.G];
        wmax = x > wmax ? x : wmax;
    }
    __syncthreads();   // R[b] written by this workgroup is read back below

    int64_t max_s = 0, max_r = 0, lb = 0, total = 0, spread = 0;
    for (int k = threadIdx.x; k < a.M; k += THREADS) {
        int64_t out = 0, in = 0, smin = INT64_MAX, smax = 0;
        for (int n = 0; n < a.N; ++n) {
            const int64_t s = Sb[k * a.N + n], r = Rb[k * a.N + n];
            out += s; in += r;
            max_s = s > max_s ? s : max_s;
            max_r = r > max_r ? r : max_r;
            smin = s < smin ? s : smin;
            smax = s > smax ? s : smax;
        }
        total += out;
        const int64_t co = (out + a.N - 1) / a.N, ci = (in + a.N - 1) / a.N;
        lb = co > lb ? co : lb;
        lb = ci > lb ? ci : lb;
        spread = (smax - smin) > spread ? (smax - smin) : spread;
    }
    // five maxima and one sum, together
    int64_t v[6] = {max_s, max_r, lb, wmax, spread, total};
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
#pragma unroll
        for (int j = 0; j < 6; ++j) {
            const int64_t o = __shfl_xor(v[j], d);
            v[j] = j == 5 ? v[j] + o : (o > v[j] ? o : v[j]);
        }
    }
    if (lane == 0)
#pragma unroll
        for (int j = 0; j < 6; ++j) sh[j][wave] = v[j];
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int j = 0; j < 6; ++j) {
            int64_t r = sh[j][0];
            for (int w = 1; w < WAVES; ++w) r = j == 5 ? r + sh[j][w] : (sh[j][w] > r ? sh[j][w] : r);
            v[j] = r;
        }
        int64_t *st = a.stats + (int64_t)b * 8;
        st[0] = v[0] > v[1] ? v[0] : v[1];
        st[1] = v[0];
        st[2] = v[1];
        st[3] = v[2] > v[3] ? v[2] : v[3];
        st[4] = v[5];
        st[5] = v[3];
        st[6] = a.chunk_off[(int64_t)(b + 1) * a.M] - a.chunk_off[(int64_t)b * a.M];
        st[7] = v[4];
    }
}

int launch_eval_reduce(const EvArgs &a, int batch, hipStream_t st)
{
    if ((int64_t)a.slices * a.G <= 16384 && a.M <= 256) {
        hipLaunchKernelGGL((eval_reduce_kernel<256, true>), dim3((unsigned)batch), dim3(256), 0, st, a);
    } else if ((int64_t)a.slices * a.G <= 131072) {
        hipLaunchKernelGGL((eval_reduce_kernel<1024, true>), dim3((unsigned)batch), dim3(1024), 0, st, a);
    } else {
        hipLaunchKernelGGL(eval_sum_kernel, dim3((unsigned)((a.G + 63) / 64), (unsigned)batch), dim3(256), 0, st, a);
        if (int rc = launch_status()) return rc;
        hipLaunchKernelGGL((eval_reduce_kernel<1024, false>), dim3((unsigned)batch), dim3(1024), 0, st, a);
    }
    return launch_status();
}

static int eval_slices(int32_t batch)
{
    // about 2048 workgroups in flight whatever the batch; at least one slice per matrix
    int s = (2048 + batch - 1) / (batch > 0 ? batch : 1);
    if (s < 1) s = 1;
    if (s > 2048) s = 2048;
    return s;
}

}  // namespace rs

extern "C" size_t railsched_eval_workspace_bytes(int32_t batch, const railsched_topo_t *h_topo)
{
    using namespace rs;
    if (check_topo(h_topo) != RAILSCHED_OK || batch < 0) return 0;
    const int64_t G = (int64_t)h_topo->nodes * h_topo->rails;
    const size_t n = sizeof(int64_t) * (size_t)batch * (size_t)eval_slices(batch) * (size_t)(G + 1);
    return n ? align_up(n, 256) : 256;
}

extern "C" int railsched_eval(const int64_t *chunk_off, const uint32_t *chunk_w, const uint32_t *chunk_flow,
                              const uint8_t *rail, const int64_t *S, int32_t batch, const railsched_topo_t *h_topo,
                              int64_t capacity, int64_t *R, int64_t *stats, void *ws, size_t ws_bytes, void *stream)
{
    using namespace rs;
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0 || capacity < 0) return RAILSCHED_ERR_INVALID_ARG;
    if (batch > 65535) return RAILSCHED_ERR_UNSUPPORTED;
    if (batch == 0) return RAILSCHED_OK;
    if (!chunk_off || !S || !R || !stats || (capacity > 0 && (!chunk_w || !chunk_flow || !rail))) return RAILSCHED_ERR_NULL_PTR;
    if (!ws || ws_bytes < railsched_eval_workspace_bytes(batch, h_topo) || reinterpret_cast<uintptr_t>(ws) % 256)
        return RAILSCHED_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);

    EvArgs a;
    a.chunk_off = chunk_off; a.chunk_w = chunk_w; a.chunk_flow = chunk_flow; a.rail = rail; a.S = S;
    a.R = R; a.stats = stats; a.partial = static_cast<int64_t *>(ws);
    a.M = h_topo->nodes; a.N = h_topo->rails; a.G = a.M * a.N; a.slices = eval_slices(batch);
    a.capacity = capacity; a.n_inst = batch * a.M;
    a.nshift = is_pow2(a.N) ? ilog2(a.N) : -1;
    a.gmask = is_pow2(a.G) ? a.G - 1 : -1;
    a.wide_ok = (reinterpret_cast<uintptr_t>(chunk_w) % 16 == 0 && reinterpret_cast<uintptr_t>(chunk_flow) % 16 == 0 &&
                 reinterpret_cast<uintptr_t>(rail) % 4 == 0) ? 1 : 0;

    a.copies = 16;
    while (a.copies > 1 && sizeof(unsigned long long) * (size_t)(a.G + 1) * a.copies > 40 * 1024) a.copies /= 2;
    const size_t lds = sizeof(unsigned long long) * (size_t)(a.G + 1) * a.copies;
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(eval_partial_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return RAILSCHED_ERR_HIP;
    }
    hipLaunchKernelGGL(eval_partial_kernel, dim3((unsigned)a.slices, (unsigned)batch), dim3(kEvThreads), lds, st, a);
    if (int rc = launch_status()) return rc;
    return launch_eval_reduce(a, batch, st);
}
