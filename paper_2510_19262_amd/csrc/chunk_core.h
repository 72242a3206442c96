// Device-side pieces of stage 3 (Section 5.1 "Flow Splitting and Atomicity"; Algorithm 2 steps 1-2) shared by
// the stage-3 kernels and by the one-call scheduler of small batches.
#pragma once

#include "common.h"

namespace rs {

struct CsArgs {
    const int64_t *D1;
    int64_t *chunk_off;
    uint32_t *chunk_w, *chunk_flow, *perm;
    int64_t capacity;
    int64_t *cnt_all, *cnt_full, *tile_off;
    uint32_t *full_start, *canon_start;
    int64_t C;
    int32_t cshift;      // >= 0 when C is a power of two
    int32_t M, N, G, NF, intra;
    int32_t n_inst;
    int32_t tile;        // full-chunk positions per fill tile
    uint8_t *rail;       // when set, the fill also writes the rails of every instance's leading run (see cs_fill_kernel)
    int32_t nmask;       // N - 1 when N is a power of two, else -1
    int32_t gmask, nshift;   // G - 1 and log2 N when G / N are powers of two, else -1
};

__device__ __forceinline__ void split_bytes(const CsArgs &a, int64_t B, uint32_t &q, uint32_t &r)
{
    if (B < 0) B = 0;
    if (a.cshift >= 0) {
        q = (uint32_t)(B >> a.cshift);
        r = (uint32_t)(B & (a.C - 1));
    } else {
        const uint64_t qq = (uint64_t)B / (uint64_t)a.C;
        q = (uint32_t)qq;
        r = (uint32_t)((uint64_t)B - qq * (uint64_t)a.C);
    }
}

// bytes of flow f of instance (b, k); 0 for destinations inside node k unless intra-node traffic is kept
__device__ __forceinline__ int64_t flow_bytes(const CsArgs &a, const int64_t *rows, int k, int f)
{
    if (!a.intra) {
        const int node = (a.gmask >= 0 && a.nshift >= 0) ? ((f & a.gmask) >> a.nshift) : (f % a.G) / a.N;   // of the destination
        if (node == k) return 0;
    }
    return rows[f];
}

// v of the lane the DPP control points at, 0 where there is none (or where row_mask switches the row off)
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ unsigned dpp_or_zero(unsigned v)
{
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);
}

// Exclusive prefix sum over the 64 lanes (and the total), all in the vector ALU: four shifted adds inside the
// rows of 16 lanes, then lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3.
__device__ __forceinline__ unsigned wave_exscan(unsigned v, unsigned &total)
{
    unsigned inc = v;
    inc += dpp_or_zero<0x111, 0xF>(inc);            // row_shr:1
    inc += dpp_or_zero<0x112, 0xF>(inc);            // row_shr:2
    inc += dpp_or_zero<0x114, 0xF>(inc);            // row_shr:4
    inc += dpp_or_zero<0x118, 0xF>(inc);            // row_shr:8
    inc += dpp_or_zero<0x142, 0xA>(inc);            // row_bcast15 into rows 1 and 3
    inc += dpp_or_zero<0x143, 0xC>(inc);            // row_bcast31 into rows 2 and 3
    total = (unsigned)__builtin_amdgcn_readlane((int)inc, 63);
    return inc - v;
}

// Ordering point between LDS accesses of the lanes of ONE wavefront.  When the wavefront is the whole
// workgroup a workgroup barrier does; when other wavefronts of the workgroup are busy elsewhere, waiting
// for the wavefront's own LDS operations is enough (LDS executes a wavefront's operations in order) and
// the asm statement keeps the compiler from moving LDS accesses across it.
template <bool ONE_WAVE_BLOCK>
__device__ __forceinline__ void lds_sync()
{
    if constexpr (ONE_WAVE_BLOCK) __syncthreads();
    else asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

// Tails (B mod C > 0) of the flows of one instance, sorted by weight descending, ties in canonical (flow) order:
// stable LSD radix sort by one wavefront in LDS, 8-bit digits over the span of key bits that differ at all,
// ranks inside a batch of 64 from ballot matching.  rem[NF] receives every flow's tail bytes, hist[256] is
// scratch, idx_a/idx_b[NF] are ping-pong arrays of flow ids; returns the array that holds the sorted ids and
// their number in nt.
template <bool ONE_WAVE_BLOCK>
__device__ __forceinline__ unsigned short *tail_sort_wave(const CsArgs &a, const int64_t *rows, int k, unsigned *rem, unsigned *hist,
                                                          unsigned short *idx_a, unsigned short *idx_b, int &nt_out)
{
    const int lane = threadIdx.x & 63;
    const unsigned long long lt = (1ull << lane) - 1ull;
    // tails in canonical order; which key bits differ at all between them
    int nt = 0;
    unsigned any1 = 0u, all1 = 0xFFFFFFFFu;
    for (int f0 = 0; f0 < a.NF; f0 += 512) {
        int64_t bytes[8];                           // eight rounds of loads in flight: one memory round trip, not eight
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int f = f0 + 64 * u + lane;
            bytes[u] = f < a.NF ? flow_bytes(a, rows, k, f) : 0;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int f = f0 + 64 * u + lane;
            if (f0 + 64 * u >= a.NF) break;         // wave-uniform
            uint32_t q = 0, r = 0;
            if (f < a.NF) { split_bytes(a, bytes[u], q, r); rem[f] = r; }
            const unsigned long long m = __ballot(r != 0);
            if (r) { idx_a[nt + __popcll(m & lt)] = (unsigned short)f; any1 |= r; all1 &= r; }
            nt += __popcll(m);
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) { any1 |= (unsigned)__shfl_xor((int)any1, d); all1 &= (unsigned)__shfl_xor((int)all1, d); }
    lds_sync<ONE_WAVE_BLOCK>();
    // bits that are equal in every key cannot change the order: sort on the span of differing bits only
    // (token payloads make tails multiples of some power of two, so the span is usually one digit wide)
    const unsigned diff = any1 ^ all1;
    const int lo_bit = diff ? __ffs((int)diff) - 1 : 0;
    const int n_pass = (nt > 1 && diff) ? (32 - __clz((int)diff) - lo_bit + 7) / 8 : 0;

    for (int pass = 0; pass < n_pass; ++pass) {
        const int shift = lo_bit + 8 * pass;
        for (int i = lane; i < 256; i += 64) hist[i] = 0;
        lds_sync<ONE_WAVE_BLOCK>();
        for (int i = lane; i < nt; i += 64) atomicAdd(&hist[255u - ((rem[idx_a[i]] >> shift) & 255u)], 1u);
        lds_sync<ONE_WAVE_BLOCK>();
        {   // exclusive scan of the 256 buckets: four per lane
            const unsigned h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
            unsigned tot;
            const unsigned ex = wave_exscan(h0 + h1 + h2 + h3, tot);
            lds_sync<ONE_WAVE_BLOCK>();
            hist[4 * lane] = ex; hist[4 * lane + 1] = ex + h0; hist[4 * lane + 2] = ex + h0 + h1; hist[4 * lane + 3] = ex + h0 + h1 + h2;
        }
        lds_sync<ONE_WAVE_BLOCK>();
        for (int i0 = 0; i0 < nt; i0 += 64) {                            // batches in order keep the sort stable
            const int i = i0 + lane;
            const bool act = i < nt;
            const unsigned short f = act ? idx_a[i] : 0;
            const unsigned d = act ? 255u - ((rem[f] >> shift) & 255u) : 0u;
            unsigned long long peers = __ballot(act);
#pragma unroll
            for (int bit = 0; bit < 8; ++bit) {
                const bool one = (d >> bit) & 1u;
                const unsigned long long bm = __ballot(act && one);
                peers &= one ? bm : ~bm;
            }
            const unsigned base = act ? hist[d] : 0u;
            if (act) idx_b[base + __popcll(peers & lt)] = f;
            lds_sync<ONE_WAVE_BLOCK>();
            if (act && (peers >> lane) == 1ull) hist[d] = base + __popcll(peers);   // highest lane of the peer set
            lds_sync<ONE_WAVE_BLOCK>();
        }
        unsigned short *t = idx_a; idx_a = idx_b; idx_b = t;
    }

    nt_out = nt;
    return idx_a;
}

// Host side of stage 3, shared by railsched_chunk_sort and the one-call scheduler (defined in chunk_sort.hip):
// validates, lays the workspace out and launches count, scan, tail sort and fill.  With `rail` set the fill also
// writes rail[i] = i mod N for the first n_full - n_full mod N positions of every instance - the greedy
// allocation of a leading run of equal weights from empty rails (Algorithm 2 step 3) in closed form.
// *args_out, if given, receives the argument block (workspace pointers included).
int cs_run(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo, int64_t *chunk_off, uint32_t *chunk_w,
           uint32_t *chunk_flow, uint32_t *perm, int64_t capacity, uint8_t *rail, void *ws, size_t ws_bytes, hipStream_t st,
           CsArgs *args_out);

}  // namespace rs
