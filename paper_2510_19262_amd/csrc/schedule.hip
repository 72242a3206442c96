// Stages 3-5 in one call (Algorithm 2 steps 1-3 and 6; Section 4.1 load matrices): chunk split and sort, LPT
// allocation, send/receive loads and statistics.  Outputs are those of railsched_chunk_sort, railsched_lpt_spray
// and railsched_eval run one after the other, bit for bit.
//
// Large batches run the kernels of the three stages, minus what stage 3 already knows: every instance starts with
// a run of n_full chunks of weight C, whose allocation from empty rails is round robin (rail = i mod N, the closed
// form behind Theorem 4's premise of equal granularity).  So the fill kernel writes those rails with the records,
// stage 4's streaming scan for the leading runs is skipped (its serial kernels start behind them), and stage 5 gets
// the leading runs' receive loads flow by flow in closed form and reads only the few chunks behind them - 13 bytes
// of HBM traffic per chunk in all instead of 27.  Small ones - up to 1024 instances of a few thousand chunks, the
// shape of one training step's MoE layers - are bound by the latency of nine dependent launches, so they take
// three: the per-instance counts (stage 3's count kernel), then ONE workgroup per instance that does everything
// the instance needs, then the per-matrix reduction of stage 5.  Inside the workgroup, wavefront 0 sorts the
// tails and runs the serial LPT chain on them - weights and rails in LDS, the chain being what bounds the time -
// while the other wavefronts write the full-chunk records, the round-robin rails of the leading run (closed
// form: from empty rails a run of one weight is rail = i mod N) and the receive loads those imply.
#include "chunk_core.h"
#include "eval_core.h"
#include "lpt_core.h"

#include <mutex>

namespace rs {

// Workspace of railsched_schedule_static: one array per GPU, part of the library's device image, so the call needs no
// allocation.  The name below is only a handle for host code; the array's device address is asked for once per device
// (static_scratch) and that address is what kernels and every other use get.
static __device__ __align__(256) unsigned char scratch[RAILSCHED_STATIC_SCRATCH_BYTES];

constexpr int kScratchDevices = 64;
static void *g_scratch_ptr[kScratchDevices];       // device address of `scratch` on each GPU, once known
static std::mutex g_scratch_mutex;

// address of the current device's copy of `scratch`; nullptr if the runtime refuses
static void *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kScratchDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;   // this device is the current one
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

void launch_cs_count(const CsArgs &a, hipStream_t st);          // chunk_sort.hip
int lpt_serial_after_leading_runs(const int64_t *chunk_off, const uint32_t *chunk_w, int64_t n_inst, int N, uint8_t *rail,
                                  int64_t *S, int64_t capacity, hipStream_t st);   // lpt_spray.hip
void cs_ws_layout(int64_t n_inst, int64_t NF, size_t off[6]);  // chunk_sort.hip

constexpr int kSsThreads = 512;         // one wavefront on the chain, seven on the records (three: 6 us more per call on 256 instances of 7 K chunks)
constexpr int kSlThreads = 256;         // closed-form receive loads of large batches
constexpr int kSsMaxInst = 1024;        // instances whose counts one workgroup adds up
constexpr int kSsMaxFlows = 2048;       // N*G of an instance held in LDS
constexpr int kSsMaxAvg = 32768;        // chunks per instance (capacity / instances) above which one workgroup is too few

struct SsArgs {
    uint8_t *rail;
    int64_t *S;
    int64_t *partial;       // stage 5 workspace: [batch][M][G + 1]
    int32_t vec_ok;
    int32_t nshift, gmask;  // >= 0 when N / G are powers of two
};

__device__ __forceinline__ int ss_dst_node(const CsArgs &a, const SsArgs &x, uint32_t flow)   // flow = n*G + dst -> dst / N
{
    if (x.gmask >= 0 && x.nshift >= 0) return (int)((flow & (uint32_t)x.gmask) >> x.nshift);
    return (int)((flow % (uint32_t)a.G) / (uint32_t)a.N);
}

template <int GW>
__global__ __launch_bounds__(kSsThreads) void ss_instance_kernel(CsArgs a, SsArgs x)
{
    extern __shared__ unsigned long long ss_lds64[];
    __shared__ int64_t sh_red[2][kSsThreads / 64];
    __shared__ unsigned sh_wmax;
    __shared__ int sh_nt, sh_sorted_in_b;                                // wavefront 0's sort result, for the others
    // LDS: bins[G] u64 | st_fs[NF+1] | st_cs[NF] | rem[NF] | hist[256] | late_w[NF+64] | idx_a[NF] idx_b[NF] u16 | late_rail[NF+64] u8
    unsigned long long *bins = ss_lds64;
    unsigned *st_fs = reinterpret_cast<unsigned *>(bins + a.G);
    unsigned *st_cs = st_fs + a.NF + 1;
    unsigned *rem = st_cs + a.NF;
    unsigned *hist = rem + a.NF;
    unsigned *late_w = hist + 256;
    unsigned short *idx_a = reinterpret_cast<unsigned short *>(late_w + a.NF + 64);
    unsigned short *idx_b = idx_a + a.NF;
    uint8_t *late_rail = reinterpret_cast<uint8_t *>(idx_b + a.NF);

    const int inst = blockIdx.x;
    const int b = inst / a.M, k = inst % a.M;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = a.N;

    // ---- wavefront 0 starts on the tails at once; the others add up the offsets (chunks of the instances before
    // this one, and of all) and stage this instance's flow starts
    int nt = 0;
    const unsigned short *sorted = idx_a;
    int64_t before = 0, total = 0;
    if (wave == 0) {
        const int64_t *rows = a.D1 + ((int64_t)b * a.G + (int64_t)k * a.N) * a.G;
        sorted = tail_sort_wave<false>(a, rows, k, rem, hist, idx_a, idx_b, nt);
        if (lane == 0) { sh_nt = nt; sh_sorted_in_b = sorted == idx_b ? 1 : 0; }
    } else {
        constexpr int T = kSsThreads - 64;
        const int t = tid - 64;
        for (int i = t; i < a.n_inst; i += T) {
            const int64_t c = a.cnt_all[i];
            total += c;
            before += i < inst ? c : 0;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) { before += __shfl_xor(before, d); total += __shfl_xor(total, d); }
        for (int i = t; i < a.G; i += T) bins[i] = 0;
        const uint32_t *fs = a.full_start + (int64_t)inst * a.NF;
        const uint32_t *cs = a.canon_start + (int64_t)inst * a.NF;
        for (int i = t; i < a.NF; i += T) { st_fs[i] = fs[i]; st_cs[i] = cs[i]; }
        if (t == 0) st_fs[a.NF] = 0xFFFFFFFFu;                           // nothing starts behind the last flow
    }
    if (lane == 0) { sh_red[0][wave] = before; sh_red[1][wave] = total; }
    const uint32_t n_full = (uint32_t)a.cnt_full[inst];
    const uint32_t n_all = (uint32_t)a.cnt_all[inst];
    __syncthreads();
    before = 0; total = 0;
#pragma unroll
    for (int w = 0; w < kSsThreads / 64; ++w) { before += sh_red[0][w]; total += sh_red[1][w]; }
    const int64_t out0 = before;
    nt = sh_nt;
    sorted = sh_sorted_in_b ? idx_b : idx_a;
    if (tid == 0) {
        a.chunk_off[inst] = out0;
        if (inst == a.n_inst - 1) a.chunk_off[a.n_inst] = total;
    }
    if (total > a.capacity) {                                            // record arrays too small: leave them alone, mark the loads
        if (tid < N) x.S[(int64_t)inst * N + tid] = -1;
        return;
    }

    // leading run: the full chunks (weight C) up to a multiple of N go round robin from empty rails
    const uint32_t cw = (uint32_t)a.C;
    const uint32_t skip = n_full - n_full % (uint32_t)N;
    const uint32_t late_full = n_full - skip;                            // full chunks left to the chain (< N)

    if (wave == 0) {
        // ---- the serial chain over [late full chunks | sorted tails]; the others write the tails' records
        for (int i = lane; i < nt; i += 64) late_w[late_full + i] = rem[sorted[i]];
        if (lane < (int)late_full) late_w[lane] = cw;
        if (lane == 0) sh_wmax = n_full ? cw : (nt ? rem[sorted[0]] : 0u);
        lds_sync<false>();
        const int64_t n_late = (int64_t)late_full + nt;
        lpt_wide_body<GW, true>(late_w, late_rail, n_late, (unsigned long long)cw * (unsigned long long)(skip / (uint32_t)N), N,
                                x.S + (int64_t)inst * N, late_w);
        lds_sync<false>();
        // rails of the late chunks to memory, and their bytes to the receive bins
        for (int i = lane; i < (int)n_late; i += 64) {
            const unsigned r = late_rail[i];
            x.rail[out0 + skip + i] = (uint8_t)r;
            const uint32_t f = i < (int)late_full ? (uint32_t)last_le<uint32_t>(st_fs, a.NF, skip + i) : (uint32_t)sorted[i - late_full];
            atomicAdd(&bins[ss_dst_node(a, x, f) * N + r], (unsigned long long)late_w[i]);
        }
    } else {
        // ---- full chunks: records, rails of the leading run, receive loads of the leading run
        const int t = tid - 64;
        constexpr int T = kSsThreads - 64;
        const int64_t tail0 = out0 + n_full;
        for (int i = t; i < nt; i += T) {
            const int f = sorted[i];
            a.chunk_w[tail0 + i] = rem[f];
            a.chunk_flow[tail0 + i] = (uint32_t)f;
            // the tail is its flow's last chunk: one before the canonical start of the next flow
            if (a.perm) a.perm[tail0 + i] = (f + 1 < a.NF ? st_cs[f + 1] : n_all) - 1u;
        }
        if (x.vec_ok) {
            const uint32_t head = (uint32_t)((4 - (out0 & 3)) & 3);      // scalar positions before the first aligned group
            const uint32_t pa = n_full < head ? n_full : head;
            const uint32_t groups = (n_full - pa) / 4;
            const uint32_t pb = pa + groups * 4;
            // lane l of a wavefront takes a group whose global index is l mod 64, so the 64 lanes store one whole
            // kilobyte on a 1 KiB boundary of each record array
            const uint32_t lead_in = (uint32_t)(((out0 + pa) >> 2) & 63);
            for (uint32_t gs = t; gs < groups + lead_in; gs += T) {
                if (gs < lead_in) continue;
                const uint32_t g = gs - lead_in;
                const uint32_t p = pa + 4 * g;
                int j = last_le<uint32_t>(st_fs, a.NF, p);
                uint32_t nxt = st_fs[j + 1];
                uint32_t base = st_cs[j] - st_fs[j];                     // canonical position = base + p
                uint32_t fl[4], pm[4], rr = 0;
                uint32_t r = x.nshift >= 0 ? (p & ((1u << x.nshift) - 1u)) : p % (uint32_t)N;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    while (p + e >= nxt) { ++j; nxt = st_fs[j + 1]; base = st_cs[j] - st_fs[j]; }
                    fl[e] = (uint32_t)j;
                    pm[e] = base + p + e;
                    rr |= r << (8 * e);
                    r = (r + 1 == (uint32_t)N) ? 0u : r + 1;
                }
                *reinterpret_cast<uint4 *>(a.chunk_w + out0 + p) = make_uint4(cw, cw, cw, cw);
                *reinterpret_cast<uint4 *>(a.chunk_flow + out0 + p) = make_uint4(fl[0], fl[1], fl[2], fl[3]);
                if (a.perm) *reinterpret_cast<uint4 *>(a.perm + out0 + p) = make_uint4(pm[0], pm[1], pm[2], pm[3]);
                if (p + 4 <= skip) {
                    *reinterpret_cast<uint32_t *>(x.rail + out0 + p) = rr;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) if (p + e < skip) x.rail[out0 + p + e] = (uint8_t)(rr >> (8 * e));
                }
            }
            const uint32_t n_edge = pa + (n_full - pb);                  // at most 6 positions outside the aligned groups
            if ((uint32_t)t < n_edge) {
                const uint32_t p = (uint32_t)t < pa ? (uint32_t)t : pb + ((uint32_t)t - pa);
                const int j = last_le<uint32_t>(st_fs, a.NF, p);
                a.chunk_w[out0 + p] = cw;
                a.chunk_flow[out0 + p] = (uint32_t)j;
                if (a.perm) a.perm[out0 + p] = st_cs[j] + (p - st_fs[j]);
                if (p < skip) x.rail[out0 + p] = (uint8_t)(p % (uint32_t)N);
            }
        } else {
            for (uint32_t p = t; p < n_full; p += T) {
                const int j = last_le<uint32_t>(st_fs, a.NF, p);
                a.chunk_w[out0 + p] = cw;
                a.chunk_flow[out0 + p] = (uint32_t)j;
                if (a.perm) a.perm[out0 + p] = st_cs[j] + (p - st_fs[j]);
                if (p < skip) x.rail[out0 + p] = (uint8_t)(p % (uint32_t)N);
            }
        }
        // receive loads of the leading run, flow by flow: positions [s, e) below `skip` take rails s mod N, s+1 mod N, ...
        for (int f = t; f < a.NF; f += T) {
            const uint32_t s = st_fs[f];
            uint32_t e = f + 1 < a.NF ? st_fs[f + 1] : n_full;
            e = e < skip ? e : skip;
            if (s >= e) continue;
            const int node = ss_dst_node(a, x, (uint32_t)f);
            for (int n = 0; n < N; ++n) {
                // positions i < v with i mod N == n number (v + N - 1 - n) / N
                const uint32_t up = (uint32_t)(N - 1 - n);
                const uint32_t c = x.nshift >= 0 ? ((e + up) >> x.nshift) - ((s + up) >> x.nshift) : (e + up) / (uint32_t)N - (s + up) / (uint32_t)N;
                if (c) atomicAdd(&bins[node * N + n], (unsigned long long)c * (unsigned long long)cw);
            }
        }
    }
    __syncthreads();
    int64_t *slot = x.partial + (int64_t)inst * (a.G + 1);               // [b][k][G + 1]
    for (int i = tid; i < a.G; i += kSsThreads) slot[i] = (int64_t)bins[i];
    if (tid == 0) slot[a.G] = (int64_t)sh_wmax;
}

// ---------------------------------------------------------------------------------------------- large batches
// S[inst*N] = length of the instance's leading run of full chunks, where stage 4's serial kernels look for it
__global__ void sl_run_end_kernel(CsArgs a, int64_t *S)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.n_inst; i += gridDim.x * blockDim.x) S[(int64_t)i * a.N] = a.cnt_full[i];
}

// Receive loads of one instance into its workspace slot [G + 1]: the leading run (positions below
// n_full - n_full mod N, rails i mod N) flow by flow in closed form, the chunks behind it from their records.
__global__ __launch_bounds__(kSlThreads) void sl_recv_kernel(CsArgs a, SsArgs x)
{
    extern __shared__ unsigned long long sl_bins[];
    if (a.chunk_off[a.n_inst] > a.capacity) return;                      // the record arrays hold nothing
    const int inst = blockIdx.x, tid = threadIdx.x, N = a.N;
    for (int i = tid; i < a.G; i += kSlThreads) sl_bins[i] = 0;
    __syncthreads();
    const uint32_t n_full = (uint32_t)a.cnt_full[inst], n_all = (uint32_t)a.cnt_all[inst];
    const uint32_t lead = n_full - n_full % (uint32_t)N;
    const uint32_t cw = (uint32_t)a.C;
    const int64_t out0 = a.chunk_off[inst];
    const uint32_t *fs = a.full_start + (int64_t)inst * a.NF;
    for (int f = tid; f < a.NF; f += kSlThreads) {
        const uint32_t s = fs[f];
        uint32_t e = f + 1 < a.NF ? fs[f + 1] : n_full;
        e = e < lead ? e : lead;
        if (s >= e) continue;
        const int node = ss_dst_node(a, x, (uint32_t)f);
        for (int n = 0; n < N; ++n) {
            // positions i < v with i mod N == n number (v + N - 1 - n) / N
            const uint32_t up = (uint32_t)(N - 1 - n);
            const uint32_t c = x.nshift >= 0 ? ((e + up) >> x.nshift) - ((s + up) >> x.nshift) : (e + up) / (uint32_t)N - (s + up) / (uint32_t)N;
            if (c) atomicAdd(&sl_bins[node * N + n], (unsigned long long)c * (unsigned long long)cw);
        }
    }
    for (uint32_t p = lead + tid; p < n_all; p += kSlThreads) {
        const unsigned r = x.rail[out0 + p];
        const int node = ss_dst_node(a, x, a.chunk_flow[out0 + p]);
        if (node < a.M && r < (unsigned)N) atomicAdd(&sl_bins[node * N + r], (unsigned long long)a.chunk_w[out0 + p]);
    }
    __syncthreads();
    int64_t *slot = x.partial + (int64_t)inst * (a.G + 1);
    for (int i = tid; i < a.G; i += kSlThreads) slot[i] = (int64_t)sl_bins[i];
    if (tid == 0) slot[a.G] = n_all ? (int64_t)a.chunk_w[out0] : 0;      // records are sorted: the first is the largest
}

template <int GW>
static int launch_ss(const CsArgs &a, const SsArgs &x, hipStream_t st)
{
    const size_t lds = sizeof(unsigned long long) * (size_t)a.G + sizeof(unsigned) * (size_t)(4 * a.NF + 1 + 256 + 64) +
                       2 * sizeof(unsigned short) * (size_t)a.NF + (size_t)a.NF + 64 + 16;
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(ss_instance_kernel<GW>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return RAILSCHED_ERR_HIP;
    }
    hipLaunchKernelGGL((ss_instance_kernel<GW>), dim3((unsigned)a.n_inst), dim3(kSsThreads), lds, st, a, x);
    return launch_status();
}

}  // namespace rs

namespace rs {
// stage 5 part of the workspace: stage 5's own slots, or one slot of G + 1 sums per instance, whichever is larger
static size_t sched_eval_bytes(int32_t batch, const railsched_topo_t *h_topo)
{
    const size_t e = railsched_eval_workspace_bytes(batch, h_topo);
    const size_t G = (size_t)h_topo->nodes * h_topo->rails;
    const size_t per_inst = align_up(sizeof(int64_t) * (size_t)batch * h_topo->nodes * (G + 1), 256);
    return e > per_inst ? e : per_inst;
}
}  // namespace rs

extern "C" size_t railsched_schedule_workspace_bytes(int32_t batch, const railsched_topo_t *h_topo)
{
    const size_t s = railsched_chunk_sort_workspace_bytes(batch, h_topo);
    const size_t e = railsched_eval_workspace_bytes(batch, h_topo);
    return (s && e) ? s + rs::sched_eval_bytes(batch, h_topo) : 0;     // both are multiples of 256
}

namespace rs {
// Stages 3-5 with the workspace already checked: ws holds railsched_schedule_workspace_bytes(batch, topo) bytes, 256-byte aligned.
static int schedule_run(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo, int64_t *chunk_off, uint32_t *chunk_w,
                        uint32_t *chunk_flow, uint32_t *perm, int64_t capacity, uint8_t *rail, int64_t *S, int64_t *R, int64_t *stats,
                        void *ws, hipStream_t st)
{
    const int64_t M = h_topo->nodes, N = h_topo->rails, G = M * N, NF = N * G;
    const int64_t n_inst = (int64_t)batch * M;
    const size_t ws_sort = railsched_chunk_sort_workspace_bytes(batch, h_topo);
    char *w8 = static_cast<char *>(ws);

    const int GW = N <= 4 ? 4 : N <= 8 ? 8 : N <= 16 ? 16 : N <= 32 ? 32 : 64;
    const unsigned w_limit = GW == 4 ? WideLimit<4>::value : GW == 8 ? WideLimit<8>::value : GW == 16 ? WideLimit<16>::value
                           : GW == 32 ? WideLimit<32>::value : WideLimit<64>::value;
    const bool small = n_inst <= kSsMaxInst && NF <= kSsMaxFlows && capacity <= n_inst * (int64_t)kSsMaxAvg &&
                       (uint64_t)h_topo->chunk_bytes <= (uint64_t)w_limit;
    SsArgs x;
    x.rail = rail; x.S = S; x.partial = reinterpret_cast<int64_t *>(w8 + ws_sort);
    x.vec_ok = 0;
    x.nshift = is_pow2(N) ? ilog2(N) : -1;
    x.gmask = is_pow2(G) ? (int32_t)G - 1 : -1;
    EvArgs e;
    e.chunk_off = chunk_off; e.chunk_w = chunk_w; e.chunk_flow = chunk_flow; e.rail = rail; e.S = S;
    e.R = R; e.stats = stats; e.partial = x.partial;
    e.M = (int32_t)M; e.N = (int32_t)N; e.G = (int32_t)G; e.slices = (int32_t)M;   // one slot per instance
    e.nshift = x.nshift; e.gmask = x.gmask; e.wide_ok = 0; e.copies = 1;
    e.capacity = capacity; e.n_inst = (int32_t)n_inst;

    if (!small) {
        CsArgs a;
        if (int rc = cs_run(D1, batch, h_topo, chunk_off, chunk_w, chunk_flow, perm, capacity, rail, w8, ws_sort, st, &a)) return rc;
        hipLaunchKernelGGL(sl_run_end_kernel, dim3((unsigned)((n_inst + 255) / 256 > 1024 ? 1024 : (n_inst + 255) / 256)), dim3(256), 0, st, a, S);
        if (int rc = launch_status()) return rc;
        if (int rc = lpt_serial_after_leading_runs(chunk_off, chunk_w, n_inst, (int)N, rail, S, capacity, st)) return rc;
        const size_t lds = sizeof(unsigned long long) * (size_t)G;
        if (lds > 48 * 1024) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(sl_recv_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds) != hipSuccess)
                return RAILSCHED_ERR_HIP;
        }
        hipLaunchKernelGGL(sl_recv_kernel, dim3((unsigned)n_inst), dim3(kSlThreads), lds, st, a, x);
        if (int rc = launch_status()) return rc;
        return launch_eval_reduce(e, batch, st);
    }

    size_t off[6];
    cs_ws_layout(n_inst, NF, off);
    CsArgs a;
    a.D1 = D1; a.chunk_off = chunk_off; a.chunk_w = chunk_w; a.chunk_flow = chunk_flow; a.perm = perm;
    a.capacity = capacity;
    a.tile = 1024;                                  // unused here
    a.cnt_all = reinterpret_cast<int64_t *>(w8 + off[0]);
    a.cnt_full = reinterpret_cast<int64_t *>(w8 + off[1]);
    a.tile_off = reinterpret_cast<int64_t *>(w8 + off[2]);
    a.full_start = reinterpret_cast<uint32_t *>(w8 + off[3]);
    a.canon_start = reinterpret_cast<uint32_t *>(w8 + off[4]);
    a.C = h_topo->chunk_bytes;
    a.cshift = is_pow2(a.C) ? ilog2(a.C) : -1;
    a.M = (int32_t)M; a.N = (int32_t)N; a.G = (int32_t)G; a.NF = (int32_t)NF; a.intra = h_topo->include_intra_node;
    a.n_inst = (int32_t)n_inst;
    a.rail = nullptr; a.nmask = -1;                 // unused by the count kernel
    a.gmask = is_pow2(G) ? (int32_t)G - 1 : -1;
    a.nshift = is_pow2(N) ? ilog2(N) : -1;
    launch_cs_count(a, st);
    if (int rc = launch_status()) return rc;

    x.vec_ok = (reinterpret_cast<uintptr_t>(chunk_w) % 16 == 0 && reinterpret_cast<uintptr_t>(chunk_flow) % 16 == 0 &&
                reinterpret_cast<uintptr_t>(perm) % 16 == 0 && reinterpret_cast<uintptr_t>(rail) % 4 == 0) ? 1 : 0;
    int rc = GW == 4 ? launch_ss<4>(a, x, st) : GW == 8 ? launch_ss<8>(a, x, st) : GW == 16 ? launch_ss<16>(a, x, st)
           : GW == 32 ? launch_ss<32>(a, x, st) : launch_ss<64>(a, x, st);
    if (rc) return rc;
    return launch_eval_reduce(e, batch, st);
}

// arguments of railsched_schedule apart from the workspace: 0 and *nothing_to_do = false when the kernels should run
static int schedule_check(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo, int64_t *chunk_off, uint32_t *chunk_w,
                          uint32_t *chunk_flow, int64_t capacity, uint8_t *rail, int64_t *S, int64_t *R, int64_t *stats,
                          bool *nothing_to_do)
{
    *nothing_to_do = false;
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0 || capacity < 0) return RAILSCHED_ERR_INVALID_ARG;
    if (batch > 65535) return RAILSCHED_ERR_UNSUPPORTED;
    const int64_t M = h_topo->nodes, N = h_topo->rails, G = M * N, NF = N * G;
    if (NF > kMaxFlows) return RAILSCHED_ERR_UNSUPPORTED;
    if ((int64_t)batch * M > 0x7FFFFFFFll / 64) return RAILSCHED_ERR_UNSUPPORTED;
    if (batch == 0) { *nothing_to_do = true; return RAILSCHED_OK; }
    if (!D1 || !chunk_off || !chunk_w || !chunk_flow || !rail || !S || !R || !stats) return RAILSCHED_ERR_NULL_PTR;
    return RAILSCHED_OK;
}
}  // namespace rs

extern "C" int railsched_schedule(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo, int64_t *chunk_off,
                                  uint32_t *chunk_w, uint32_t *chunk_flow, uint32_t *perm, int64_t capacity, uint8_t *rail,
                                  int64_t *S, int64_t *R, int64_t *stats, void *ws, size_t ws_bytes, void *stream)
{
    using namespace rs;
    bool nothing = false;
    if (int rc = schedule_check(D1, batch, h_topo, chunk_off, chunk_w, chunk_flow, capacity, rail, S, R, stats, &nothing)) return rc;
    if (nothing) return RAILSCHED_OK;
    if (!ws || ws_bytes < railsched_schedule_workspace_bytes(batch, h_topo) || reinterpret_cast<uintptr_t>(ws) % 256)
        return RAILSCHED_ERR_WORKSPACE;
    return schedule_run(D1, batch, h_topo, chunk_off, chunk_w, chunk_flow, perm, capacity, rail, S, R, stats, ws,
                        static_cast<hipStream_t>(stream));
}

extern "C" int railsched_schedule_static(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo, int64_t *chunk_off,
                                         uint32_t *chunk_w, uint32_t *chunk_flow, uint32_t *perm, int64_t capacity, uint8_t *rail,
                                         int64_t *S, int64_t *R, int64_t *stats, void *stream)
{
    using namespace rs;
    bool nothing = false;
    if (int rc = schedule_check(D1, batch, h_topo, chunk_off, chunk_w, chunk_flow, capacity, rail, S, R, stats, &nothing)) return rc;
    if (nothing) return RAILSCHED_OK;
    const size_t need = railsched_schedule_workspace_bytes(batch, h_topo);
    if (need == 0 || need > (size_t)RAILSCHED_STATIC_SCRATCH_BYTES) return RAILSCHED_ERR_SCRATCH;
    void *ws = static_scratch();
    if (!ws) return RAILSCHED_ERR_HIP;
    // every word of the workspace that a kernel reads was written earlier in the same call (counts and scans by the count
    // and scan kernels, one slot of receive loads per instance or slice), so what the last call left needs no clearing
    return schedule_run(D1, batch, h_topo, chunk_off, chunk_w, chunk_flow, perm, capacity, rail, S, R, stats, ws,
                        static_cast<hipStream_t>(stream));
}
