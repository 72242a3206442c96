// Stage 3: flow splitting into fixed-size chunks and the per-node descending sort
// (Section 5.1 "Flow Splitting and Atomicity"; Algorithm 2 steps 1-2).
//
// The sorted order has structure the kernels use instead of sorting every chunk: a flow of B bytes
// gives floor(B/C) chunks of exactly C bytes and at most one tail of B mod C < C bytes.  Under
// "weight descending, ties in canonical order" all full chunks therefore come first, in canonical
// order (their positions follow from an exclusive scan of floor(B/C) over the instance's flows), and
// only the tails - at most one per flow, N*G per instance - need a real sort.  The tails of one
// instance are sorted by one wavefront with a stable LSD radix sort held in LDS (8-bit digits,
// ranks inside a 64-element batch from ballot matching).  Every chunk record is written to HBM
// exactly once.
//
// An instance (matrix b, node k) owns the N consecutive rows k*N..k*N+N-1 of D1[b]; read as one
// array of N*G entries its index is exactly the canonical flow id n*G + dst.
#include "common.h"
#include "chunk_core.h"

namespace rs {

constexpr int kTileMin = 1024;      // full-chunk positions per fill tile: a power of two between these two, chosen per call
constexpr int kTileMax = 16384;     // so that small batches still spread over a few thousand workgroups
constexpr int kFillThreads = 256;
constexpr int kFillStage = 2048;    // flow boundaries staged in LDS per span (16 KiB with the canonical starts: 8 workgroups per CU)
constexpr int kFillBlocks = 16384;  // most workgroups of one fill launch: several rounds of the chip, which evens out their ends

// ---- A: per-instance chunk counts and the two exclusive scans over its flows -----------------
__global__ __launch_bounds__(64) void cs_count_kernel(CsArgs a)
{
    const int inst = blockIdx.x;
    const int b = inst / a.M, k = inst % a.M;
    const int lane = threadIdx.x;
    const int64_t *rows = a.D1 + ((int64_t)b * a.G + (int64_t)k * a.N) * a.G;
    uint32_t *fs = a.full_start + (int64_t)inst * a.NF;
    uint32_t *cs = a.canon_start + (int64_t)inst * a.NF;
    unsigned carry_full = 0, carry_all = 0;
    int64_t n_full = 0, n_all = 0;
    for (int f0 = 0; f0 < a.NF; f0 += 256) {
        int64_t bytes[4];                           // four rounds of loads in flight before the scans, which chain
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int f = f0 + 64 * u + lane;
            bytes[u] = f < a.NF ? flow_bytes(a, rows, k, f) : 0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int f = f0 + 64 * u + lane;
            if (f0 + 64 * u >= a.NF) break;         // wave-uniform
            uint32_t q = 0, r = 0;
            if (f < a.NF) split_bytes(a, bytes[u], q, r);
            const unsigned c = q + (r ? 1u : 0u);
            unsigned tq, tc;
            const unsigned eq = wave_exscan(q, tq);
            const unsigned ec = wave_exscan(c, tc);
            if (f < a.NF) { fs[f] = carry_full + eq; cs[f] = carry_all + ec; }
            carry_full += tq; carry_all += tc;
            n_full += q; n_all += c;
        }
    }
    // exact 64-bit totals
    for (int d = 32; d >= 1; d >>= 1) { n_full += __shfl_xor(n_full, d); n_all += __shfl_xor(n_all, d); }
    if (lane == 0) { a.cnt_all[inst] = n_all; a.cnt_full[inst] = n_full; }
}

// ---- B: chunk_off = exclusive scan of instance sizes; tile_off = exclusive scan of fill tiles --
__global__ __launch_bounds__(1024) void cs_scan_kernel(CsArgs a)
{
    constexpr int PER = 4;                            // consecutive instances per thread and round
    __shared__ int64_t sh_a[16], sh_t[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile_shift = __builtin_ctz((unsigned)a.tile);   // the tile is a power of two
    int64_t carry_a = 0, carry_t = 0;                 // the same in every thread
    for (int base = 0; base < a.n_inst; base += 1024 * PER) {
        int64_t va[PER], vt[PER], sa = 0, st = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int i = base + tid * PER + u;
            va[u] = i < a.n_inst ? a.cnt_all[i] : 0;
            vt[u] = i < a.n_inst ? (a.cnt_full[i] + a.tile - 1) >> tile_shift : 0;
            sa += va[u]; st += vt[u];
        }
        int64_t ia = sa, it = st;                     // inclusive scans of the thread sums inside the wavefront
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int64_t xa = __shfl_up(ia, d), xt = __shfl_up(it, d);
            if (lane >= d) { ia += xa; it += xt; }
        }
        __syncthreads();                              // the round before is done with sh_a / sh_t
        if (lane == 63) { sh_a[wave] = ia; sh_t[wave] = it; }
        __syncthreads();
        int64_t before_a = 0, before_t = 0, tot_a = 0, tot_t = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int64_t xa = sh_a[w], xt = sh_t[w];
            if (w < wave) { before_a += xa; before_t += xt; }
            tot_a += xa; tot_t += xt;
        }
        int64_t oa = carry_a + before_a + ia - sa, ot = carry_t + before_t + it - st;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int i = base + tid * PER + u;
            if (i < a.n_inst) { a.chunk_off[i] = oa; a.tile_off[i] = ot; }
            oa += va[u]; ot += vt[u];
        }
        carry_a += tot_a; carry_t += tot_t;
    }
    if (tid == 0) { a.chunk_off[a.n_inst] = carry_a; a.tile_off[a.n_inst] = carry_t; }
}

// ---- C: tails of one instance: stable descending radix sort in LDS, one wavefront -------------
__global__ __launch_bounds__(64) void cs_tail_kernel(CsArgs a)
{
    extern __shared__ unsigned cs_lds[];
    unsigned *rem = cs_lds;                                              // [NF] tail bytes per flow
    unsigned *hist = cs_lds + a.NF;                                      // [256]
    unsigned short *idx_a = reinterpret_cast<unsigned short *>(hist + 256);   // [NF] flow ids, ping
    unsigned short *idx_b = idx_a + a.NF;                                      // [NF] pong
    if (a.chunk_off[a.n_inst] > a.capacity) return;                      // record arrays too small: leave them alone

    const int inst = blockIdx.x;
    const int b = inst / a.M, k = inst % a.M;
    const int lane = threadIdx.x;
    const int64_t *rows = a.D1 + ((int64_t)b * a.G + (int64_t)k * a.N) * a.G;

    int nt = 0;
    unsigned short *sorted = tail_sort_wave<true>(a, rows, k, rem, hist, idx_a, idx_b, nt);
    idx_a = sorted;

    const int64_t out0 = a.chunk_off[inst] + a.cnt_full[inst];
    const uint32_t *cs = a.canon_start + (int64_t)inst * a.NF;
    const uint32_t n_all = (uint32_t)a.cnt_all[inst];
    for (int i = lane; i < nt; i += 64) {
        const int f = idx_a[i];
        a.chunk_w[out0 + i] = rem[f];
        a.chunk_flow[out0 + i] = (uint32_t)f;
        // the tail is its flow's last chunk: one before the canonical start of the next flow
        if (a.perm) a.perm[out0 + i] = (f + 1 < a.NF ? cs[f + 1] : n_all) - 1u;
    }
}

// ---- D: full chunks: tiles of consecutive output positions ------------------------------------
// Full-chunk region of the instances, cut into tiles of a.tile positions; a workgroup takes a contiguous run of
// tiles, so the instance and the flow its next tile starts in carry over and only its first tile is searched for.
// A tile is filled in spans: as many flow boundaries as fit are staged in LDS (in rounds of 512, until they reach
// the tile's end), and the span ends where the staged flows end.  Inside a span positions are grouped by fours at
// multiples of four of the global record index (16-byte stores); a wavefront walks a contiguous quarter of the
// groups, 64 at a time, so the flow of its first group is known from the step before, one ballot over the next 64
// boundaries bounds the flows its 256 positions can lie in, and each lane finishes with a binary search over that
// handful.
__global__ __launch_bounds__(kFillThreads) void cs_fill_kernel(CsArgs a, int vec_ok)
{
    __shared__ uint32_t st_fs[kFillStage + 1];
    __shared__ uint32_t st_cs[kFillStage];
    if (a.chunk_off[a.n_inst] > a.capacity) return;
    const int64_t n_tiles = a.tile_off[a.n_inst];
    const int64_t u0 = n_tiles * blockIdx.x / gridDim.x, u1 = n_tiles * (blockIdx.x + 1) / gridDim.x;
    if (u0 >= u1) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int kWaves = kFillThreads / 64;
    const uint32_t cw = (uint32_t)a.C;

    int inst = wave_last_le<int64_t>(a.tile_off, a.n_inst, u0);          // tile_off[inst] <= u0 < tile_off[inst+1]
    int64_t t_end = a.tile_off[inst + 1];
    int fb = -1;                                                         // flow that holds the position before the next span
    for (int64_t u = u0; u < u1; ++u) {
        if (u >= t_end) {
            do { ++inst; t_end = a.tile_off[inst + 1]; } while (u >= t_end);
            fb = -1;
        }
        const uint32_t n_full = (uint32_t)a.cnt_full[inst];
        const uint32_t t0 = (uint32_t)(u - a.tile_off[inst]) * (uint32_t)a.tile;
        const uint32_t t1 = (n_full - t0 < (uint32_t)a.tile) ? n_full : t0 + (uint32_t)a.tile;
        const uint32_t *fs = a.full_start + (int64_t)inst * a.NF;
        const uint32_t *cs = a.canon_start + (int64_t)inst * a.NF;
        const int64_t out0 = a.chunk_off[inst];
        const uint32_t lead = n_full - n_full % (uint32_t)a.N;          // positions below it go round robin (a.rail)
        if (fb < 0) fb = wave_last_le<uint32_t>(fs, a.NF, t0);

        uint32_t p0 = t0;
        while (p0 < t1) {
            // ---- stage flow starts fb.. until they pass the tile's end, the flows end or the stage is full
            __syncthreads();                                             // the span before is done with the stage
            int nf = 0;
            bool covers = false;
            while (true) {
                int want = a.NF - fb - nf;
                want = want < 512 ? want : 512;
                want = want < kFillStage - nf ? want : kFillStage - nf;
                for (int i = threadIdx.x; i < want; i += kFillThreads) {
                    st_fs[nf + i] = fs[fb + nf + i];
                    if (a.perm) st_cs[nf + i] = cs[fb + nf + i];
                }
                __syncthreads();
                nf += want;
                covers = (fb + nf >= a.NF) || (st_fs[nf - 1] >= t1);
                if (covers || nf >= kFillStage) break;
            }
            // the span ends at the tile's end, or where the last staged flow starts (it may continue unstaged)
            uint32_t p1 = t1;
            if (!covers) {
                p1 = st_fs[nf - 1];
                if (p1 <= p0) { fb += nf - 1; continue; }                // a stage full of empty flows: move on in the flows
            }
            __syncthreads();                                             // everyone has read st_fs[nf-1]
            if (threadIdx.x == 0) st_fs[nf] = 0xFFFFFFFFu;               // nothing starts behind the staged flows
            __syncthreads();

            if (vec_ok) {
                const uint32_t head = (uint32_t)((4 - ((out0 + p0) & 3)) & 3);   // scalar positions before the first aligned group
                const uint32_t pa = (p1 - p0 < head) ? p1 : p0 + head;
                const uint32_t groups = (p1 - pa) / 4;
                const uint32_t pb = pa + groups * 4;                              // scalar positions from here on
                // The wavefronts' shares and their steps end on 1 KiB boundaries of the record arrays (64 groups), so all
                // steps but the span's first and last store whole, aligned kilobytes: 10 % more write rate than
                // kilobytes that start 16 bytes off.
                const uint32_t G0 = (uint32_t)(((out0 + pa) >> 2) & 63);           // global group index of group 0, mod 64
                auto share = [&](int w) {
                    if (w <= 0) return 0u;
                    if (w >= kWaves) return groups;
                    const uint32_t cut = ((G0 + (uint32_t)((uint64_t)groups * w / kWaves)) & ~63u);
                    return cut > G0 ? cut - G0 : 0u;
                };
                const uint32_t g0 = share(wave), g1 = share(wave + 1);
                if (g0 < g1) {
                    int j_lo = last_le<uint32_t>(st_fs, nf, pa + 4 * g0);          // the same in every lane
                    uint32_t cnt = 0;
                    for (uint32_t gb = g0; gb < g1; gb += cnt) {
                        cnt = 64u - ((G0 + gb) & 63u);
                        cnt = cnt < g1 - gb ? cnt : g1 - gb;
                        const bool active = (uint32_t)lane < cnt;
                        const uint32_t g = active ? gb + lane : gb + cnt - 1;      // idle lanes shadow the step's last group
                        const uint32_t p = pa + 4 * g;
                        const uint32_t g_last = gb + cnt - 1;
                        const uint32_t p_last = pa + 4 * g_last + 3;
                        // boundaries j_lo+1 .. j_lo+64: those at or below the step's last position form a prefix
                        const int probe = j_lo + 1 + lane;
                        const uint32_t pv = probe <= nf ? st_fs[probe] : 0xFFFFFFFFu;
                        const int inside = __popcll(__ballot(pv <= p_last));
                        int lo = j_lo, hi = inside < 64 ? j_lo + inside + 1 : nf;   // flow of p lies in [lo, hi)
                        while (hi - lo > 1) {
                            const int mid = (lo + hi) >> 1;
                            if (st_fs[mid] <= p) lo = mid; else hi = mid;
                        }
                        int j = lo;
                        uint32_t nxt = st_fs[j + 1];
                        uint32_t base = a.perm ? st_cs[j] - st_fs[j] : 0u;       // canonical position = base + p
                        uint32_t fl[4], pm[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            while (p + e >= nxt) {
                                ++j;
                                nxt = st_fs[j + 1];
                                base = a.perm ? st_cs[j] - st_fs[j] : 0u;
                            }
                            fl[e] = (uint32_t)(fb + j);
                            pm[e] = base + p + e;
                        }
                        if (active && a.rail) {                      // leading run: rail = position mod N
                            uint32_t r = a.nmask >= 0 ? (p & (uint32_t)a.nmask) : p % (uint32_t)a.N, rr = 0;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                rr |= r << (8 * e);
                                r = (r + 1 == (uint32_t)a.N) ? 0u : r + 1;
                            }
                            if (p + 4 <= lead) {
                                *reinterpret_cast<uint32_t *>(a.rail + out0 + p) = rr;
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; ++e) if (p + e < lead) a.rail[out0 + p + e] = (uint8_t)(rr >> (8 * e));
                            }
                        }
                        if (active) {
                            *reinterpret_cast<uint4 *>(a.chunk_w + out0 + p) = make_uint4(cw, cw, cw, cw);
                            *reinterpret_cast<uint4 *>(a.chunk_flow + out0 + p) = make_uint4(fl[0], fl[1], fl[2], fl[3]);
                            if (a.perm) *reinterpret_cast<uint4 *>(a.perm + out0 + p) = make_uint4(pm[0], pm[1], pm[2], pm[3]);
                        }
                        j_lo = __builtin_amdgcn_readlane(j, 63);         // flow of the step's last position
                    }
                }
                // the few positions before the first and behind the last aligned group
                const uint32_t n_edge = (pa - p0) + (p1 - pb);
                if (threadIdx.x < n_edge) {
                    const uint32_t p = threadIdx.x < pa - p0 ? p0 + threadIdx.x : pb + (threadIdx.x - (pa - p0));
                    const int j = last_le<uint32_t>(st_fs, nf, p);
                    a.chunk_w[out0 + p] = cw;
                    a.chunk_flow[out0 + p] = (uint32_t)(fb + j);
                    if (a.perm) a.perm[out0 + p] = st_cs[j] + (p - st_fs[j]);
                    if (a.rail && p < lead) a.rail[out0 + p] = (uint8_t)(p % (uint32_t)a.N);
                }
            } else {
                for (uint32_t p = p0 + threadIdx.x; p < p1; p += kFillThreads) {
                    const int j = last_le<uint32_t>(st_fs, nf, p);
                    a.chunk_w[out0 + p] = cw;
                    a.chunk_flow[out0 + p] = (uint32_t)(fb + j);
                    if (a.perm) a.perm[out0 + p] = st_cs[j] + (p - st_fs[j]);
                    if (a.rail && p < lead) a.rail[out0 + p] = (uint8_t)(p % (uint32_t)a.N);
                }
            }
            // the next span starts in the flow that holds position p1 - 1
            fb += last_le<uint32_t>(st_fs, nf, p1 - 1);
            p0 = p1;
        }
    }
}

static void ws_layout(int64_t n_inst, int64_t NF, size_t off[6])
{
    size_t o = 0;
    off[0] = o; o += align_up(sizeof(int64_t) * (size_t)n_inst, 256);          // cnt_all
    off[1] = o; o += align_up(sizeof(int64_t) * (size_t)n_inst, 256);          // cnt_full
    off[2] = o; o += align_up(sizeof(int64_t) * (size_t)(n_inst + 1), 256);    // tile_off
    off[3] = o; o += align_up(sizeof(uint32_t) * (size_t)(n_inst * NF), 256);  // full_start
    off[4] = o; o += align_up(sizeof(uint32_t) * (size_t)(n_inst * NF), 256);  // canon_start
    off[5] = o;
}

// entry points for the one-call scheduler (schedule.hip)
void cs_ws_layout(int64_t n_inst, int64_t NF, size_t off[6]) { ws_layout(n_inst, NF, off); }
void launch_cs_count(const CsArgs &a, hipStream_t st)
{
    hipLaunchKernelGGL(cs_count_kernel, dim3((unsigned)a.n_inst), dim3(64), 0, st, a);
}

}  // namespace rs

extern "C" size_t railsched_chunk_sort_workspace_bytes(int32_t batch, const railsched_topo_t *h_topo)
{
    using namespace rs;
    if (check_topo(h_topo) != RAILSCHED_OK || batch < 0) return 0;
    const int64_t G = (int64_t)h_topo->nodes * h_topo->rails;
    size_t off[6];
    ws_layout((int64_t)batch * h_topo->nodes, (int64_t)h_topo->rails * G, off);
    return off[5] ? off[5] : 256;
}

namespace rs {
int cs_run(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo, int64_t *chunk_off, uint32_t *chunk_w,
           uint32_t *chunk_flow, uint32_t *perm, int64_t capacity, uint8_t *rail, void *ws, size_t ws_bytes, hipStream_t st,
           CsArgs *args_out)
{
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0 || capacity < 0) return RAILSCHED_ERR_INVALID_ARG;
    const int64_t M = h_topo->nodes, N = h_topo->rails, G = M * N, NF = N * G;
    if (NF > kMaxFlows) return RAILSCHED_ERR_UNSUPPORTED;
    const int64_t n_inst = (int64_t)batch * M;
    if (n_inst > 0x7FFFFFFFll) return RAILSCHED_ERR_UNSUPPORTED;
    if (!chunk_off) return RAILSCHED_ERR_NULL_PTR;
    if (n_inst > 0 && !D1) return RAILSCHED_ERR_NULL_PTR;
    if (chunk_w && !chunk_flow) return RAILSCHED_ERR_NULL_PTR;
    size_t off[6];
    ws_layout(n_inst, NF, off);
    if (!ws || ws_bytes < off[5] || reinterpret_cast<uintptr_t>(ws) % 256) return RAILSCHED_ERR_WORKSPACE;
    char *w8 = static_cast<char *>(ws);
    CsArgs a;
    a.D1 = D1; a.chunk_off = chunk_off; a.chunk_w = chunk_w; a.chunk_flow = chunk_flow; a.perm = perm;
    a.capacity = capacity;
    a.tile = kTileMin;
    while (a.tile < kTileMax && capacity / a.tile > 8192) a.tile *= 2;
    a.cnt_all = reinterpret_cast<int64_t *>(w8 + off[0]);
    a.cnt_full = reinterpret_cast<int64_t *>(w8 + off[1]);
    a.tile_off = reinterpret_cast<int64_t *>(w8 + off[2]);
    a.full_start = reinterpret_cast<uint32_t *>(w8 + off[3]);
    a.canon_start = reinterpret_cast<uint32_t *>(w8 + off[4]);
    a.C = h_topo->chunk_bytes;
    a.cshift = is_pow2(a.C) ? ilog2(a.C) : -1;
    a.M = (int32_t)M; a.N = (int32_t)N; a.G = (int32_t)G; a.NF = (int32_t)NF; a.intra = h_topo->include_intra_node;
    a.n_inst = (int32_t)n_inst;
    a.rail = rail;
    a.nmask = is_pow2(N) ? (int32_t)N - 1 : -1;
    a.gmask = is_pow2(G) ? (int32_t)G - 1 : -1;
    a.nshift = is_pow2(N) ? ilog2(N) : -1;
    if (args_out) *args_out = a;

    if (n_inst > 0) {
        hipLaunchKernelGGL(cs_count_kernel, dim3((unsigned)n_inst), dim3(64), 0, st, a);
        if (int rc = launch_status()) return rc;
    }
    hipLaunchKernelGGL(cs_scan_kernel, dim3(1), dim3(1024), 0, st, a);
    if (int rc = launch_status()) return rc;
    if (!chunk_w || n_inst == 0) return RAILSCHED_OK;

    const size_t lds = sizeof(unsigned) * (size_t)(NF + 256) + 2 * sizeof(unsigned short) * (size_t)NF;
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(cs_tail_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return RAILSCHED_ERR_HIP;
    }
    hipLaunchKernelGGL(cs_tail_kernel, dim3((unsigned)n_inst), dim3(64), lds, st, a);
    if (int rc = launch_status()) return rc;
    const int vec_ok = (reinterpret_cast<uintptr_t>(chunk_w) % 16 == 0 && reinterpret_cast<uintptr_t>(chunk_flow) % 16 == 0 &&
                        reinterpret_cast<uintptr_t>(perm) % 16 == 0 && reinterpret_cast<uintptr_t>(rail) % 4 == 0) ? 1 : 0;
    // no launch needs more workgroups than there can be tiles: capacity/tile full ones and one ragged one per instance
    int64_t fill_blocks = capacity / a.tile + n_inst;
    fill_blocks = fill_blocks < 1 ? 1 : fill_blocks > kFillBlocks ? kFillBlocks : fill_blocks;
    hipLaunchKernelGGL(cs_fill_kernel, dim3((unsigned)fill_blocks), dim3(kFillThreads), 0, st, a, vec_ok);
    return launch_status();
}
}  // namespace rs

extern "C" int railsched_chunk_sort(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo,
                                    int64_t *chunk_off, uint32_t *chunk_w, uint32_t *chunk_flow, uint32_t *perm,
                                    int64_t capacity, void *ws, size_t ws_bytes, void *stream)
{
    return rs::cs_run(D1, batch, h_topo, chunk_off, chunk_w, chunk_flow, perm, capacity, nullptr, ws, ws_bytes,
                      static_cast<hipStream_t>(stream), nullptr);
}
