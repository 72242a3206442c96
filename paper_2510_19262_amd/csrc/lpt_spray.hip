// Stage 4: LPT iterative allocation (Algorithm 2, initialisation and step 3).
//
// The loop is serial inside one (matrix, node) instance - every decision depends on all earlier
// ones - and independent across instances.  LoadState lives in lanes: a group of GW = 2^S lanes
// (GW >= N) holds the N rail loads, lane q holds rail q.  Per chunk the group needs
//   j* = lowest-numbered rail of minimum load,   LoadState[j*] += w.
//
// Packed keys.  Greedy assignment keeps max(LoadState) - min(LoadState) <= the largest weight seen so
// far (the fullest rail was the emptiest one just before its last chunk).  Loads are therefore kept
// as a 64-bit base shared by the group plus a small per-lane delta, and the lane packs
// key = (delta << S) | q into 32 bits: one unsigned min over the group, done with DPP exchanges,
// yields both the minimum and the lowest rail index that attains it, and key equality marks the
// winner.  The base is advanced after every period so deltas stay small.
// Exact path.  As soon as a weight above the packing limit shows up, the wave switches for good to
// plain 64-bit loads with an explicit (load, rail) lexicographic reduction.  Both compute the same
// function; the loads that leave the kernel are exact 64-bit sums.
// Runs.  Chunk lists are dominated by long runs of one weight (every full chunk weighs C).  A period
// of equal weights that starts from loads within one weight of each other needs no chain at all (see
// closed_period below).  railsched_lpt_spray uses that shortcut, railsched_lpt_spray_chunkwise never
// does; their outputs are identical.
//
// Leading run.  From empty rails a run of one weight w > 0 is pure round robin: chunk i goes to rail
// i mod N whatever happened elsewhere, so it needs no state and is written by a streaming kernel over
// all chunks of all instances at once (lpt_prefix_kernel), which also finds, per instance, where the
// run ends.  The serial kernels then start behind it with the closed-form loads.
//
// Three launch shapes (the third, "rows", four instances per wavefront in the sorted form, sits between the two
// described here and has its own comment further down).  "Packed": 64/GW instances share a wavefront, one per lane group, so one
// instruction stream advances several schedulers - the shape for tens of thousands of instances,
// where issue slots are the limit.  "Wide": one instance per wavefront, its state replicated in
// every row of lanes, all 64 lanes streaming weights and writing rails - the shape for few instances,
// where the latency of the chain and of HBM is the limit and more wavefronts hide more of it.  The
// wide shape keeps the keys sorted across lanes instead of by rail (lpt_core.h): the argmin is then
// always in lane 0 and a step is a subtraction and a median of three.
// With a workspace a packed launch orders its instances by length and gives the few longest the wide shape.
#include "common.h"
#include "chunk_core.h"
#include "lpt_core.h"

namespace rs {

// ================================================================================ leading run
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kPfThreads = 256;
constexpr int kPfTile = 16384;      // most chunk positions per workgroup iteration (16 x uint4 per thread)
constexpr int kPfPass = kPfThreads * 4;   // positions one pass of the workgroup covers
constexpr int kPfStage = 1024;      // instance boundaries staged in LDS per tile
constexpr int kPfBlocks = 16384;   // short-lived workgroups stream best (2048: 12 % slower on long lists); more cost short lists their empty launches
constexpr int kPfRun = 4;           // consecutive tiles a workgroup takes at a time

__global__ void lpt_prefix_init_kernel(int64_t *run_end, int n_inst, int N)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_inst; i += gridDim.x * blockDim.x) run_end[(int64_t)i * N] = INT64_MAX;
}

// Every chunk position p of every instance: rail[p] = (position inside the instance) mod N, and
// run_end[inst*N] = min(position inside the instance of the first weight that differs from the
// instance's first weight).  Positions are handled four at a time at multiples of four, so weights
// load as 16 bytes and rails store as 4 bytes whatever the instance offsets are.  run_end lives in the
// first slot of the instance's S row, which the serial kernel overwrites with the loads afterwards.
__global__ __launch_bounds__(kPfThreads) void lpt_prefix_kernel(const int64_t *__restrict__ chunk_off,
                                                                const uint32_t *__restrict__ chunk_w, int n_inst, int N,
                                                                int nmask, uint8_t *__restrict__ rail, int64_t *run_end,
                                                                int wide_ok, int64_t capacity)
{
    __shared__ int64_t s_off[kPfStage + 1];
    __shared__ uint32_t s_w0[kPfStage];
    const int64_t total = chunk_off[n_inst];
    if (total > capacity) return;                   // more chunks than the arrays hold: the serial kernel marks S
    // tile: the share of one workgroup when the whole grid takes one tile each, in whole passes, at most kPfTile
    int64_t tile = ((total + gridDim.x - 1) / gridDim.x + kPfPass - 1) / kPfPass * kPfPass;
    tile = tile < kPfPass ? kPfPass : tile > kPfTile ? kPfTile : tile;
    // A workgroup takes up to kPfRun consecutive tiles at a time: the instance a tile starts in is searched for once per run
    // and carried from tile to tile (each search is two or three dependent trips to memory, a fifth of the time a
    // workgroup spent on a tile when every tile searched for both of its ends).
    int64_t run = total / ((int64_t)gridDim.x * tile);     // short lists keep one tile per workgroup: parallelism first
    run = run < 1 ? 1 : run > kPfRun ? kPfRun : run;
    const int64_t span = tile * run;
    for (int64_t s0 = (int64_t)blockIdx.x * span; s0 < total; s0 += (int64_t)gridDim.x * span) {
        const int64_t s1 = s0 + span < total ? s0 + span : total;
        int inst_lo = wave_last_le<int64_t>(chunk_off, n_inst, s0);
        for (int64_t t0 = s0; t0 < s1; t0 += tile) {
            const int64_t t1 = t0 + tile < s1 ? t0 + tile : s1;
            int64_t next_off = chunk_off[inst_lo + 1];
            for (int hops = 0; next_off <= t0; ++hops) {       // on to the instance that holds t0 (empty ones are skipped)
                if (hops == 8) { inst_lo = wave_last_le<int64_t>(chunk_off, n_inst, t0); next_off = chunk_off[inst_lo + 1]; break; }
                ++inst_lo;
                next_off = chunk_off[inst_lo + 1];
            }
            const bool one = next_off >= t1;                   // the tile lies inside instance inst_lo
            const int inst_hi = one ? inst_lo : wave_last_le<int64_t>(chunk_off, n_inst, t1 - 1);
            const int cnt = inst_hi - inst_lo + 1;
            const bool fast = one && wide_ok && ((t1 - t0) & 3) == 0;
            const bool staged = cnt <= kPfStage;
            if (!fast) {
                __syncthreads();                               // previous tile is done with the stage
                if (staged) {
                    for (int i = threadIdx.x; i <= cnt; i += kPfThreads) s_off[i] = chunk_off[inst_lo + i];
                    for (int i = threadIdx.x; i < cnt; i += kPfThreads) {
                        const int64_t b = chunk_off[inst_lo + i];
                        s_w0[i] = b < total ? chunk_w[b] : 0u;  // an empty instance's value is never used
                    }
                }
                __syncthreads();
            }
            if (fast) {
                // The tile lies inside one instance (the common case when instances are long): four 16-byte loads
                // in flight per thread, one comparison per weight, and one atomic per wavefront at most.
                const int64_t b = chunk_off[inst_lo];
                const uint32_t w0 = chunk_w[b];
                int64_t miss = INT64_MAX;
                constexpr int U = 4;
                // memory operations of a wavefront complete in order, so the loads of the next step are issued ahead of
                // this step's stores instead of behind them
                int64_t p = t0 + (int64_t)threadIdx.x * 4;
                u32x4 v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t pu = p + (int64_t)u * kPfThreads * 4;
                    v[u] = pu < t1 ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(chunk_w + pu)) : u32x4{w0, w0, w0, w0};
                }
                while (p < t1) {
                    uint32_t packed[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int64_t i = p + (int64_t)u * kPfThreads * 4 - b;
                        uint32_t r0 = nmask >= 0 ? ((uint32_t)i & (uint32_t)nmask) : (uint32_t)((uint64_t)i % (uint64_t)N);
                        packed[u] = r0;
#pragma unroll
                        for (int e = 1; e < 4; ++e) {
                            r0 = (r0 + 1 == (uint32_t)N) ? 0u : r0 + 1;
                            packed[u] |= r0 << (8 * e);
                        }
                        const int first = v[u].x != w0 ? 0 : v[u].y != w0 ? 1 : v[u].z != w0 ? 2 : v[u].w != w0 ? 3 : -1;
                        if (first >= 0 && i + first < miss) miss = i + first;          // padded lanes hold w0: never a miss
                    }
                    const int64_t pn = p + (int64_t)kPfThreads * 4 * U;
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int64_t pu = pn + (int64_t)u * kPfThreads * 4;
                        v[u] = pu < t1 ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(chunk_w + pu)) : u32x4{w0, w0, w0, w0};
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int64_t pu = p + (int64_t)u * kPfThreads * 4;
                        if (pu < t1) __builtin_nontemporal_store(packed[u], reinterpret_cast<uint32_t *>(rail + pu));
                    }
                    p = pn;
                }
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) { const int64_t o = __shfl_xor(miss, d); miss = o < miss ? o : miss; }
                if ((threadIdx.x & 63) == 0 && miss != INT64_MAX) {
                    const int64_t slot = (int64_t)inst_lo * N;
                    if (run_end[slot] > miss) atomicMin((long long *)&run_end[slot], (long long)miss);
                }
                continue;
            }
            // The general sweep, once for boundaries staged in LDS and once for boundaries read from memory: through
            // one pointer that may be either, every lookup was a flat load, which waits for all of the wavefront's
            // memory traffic.  offs[i] = start of instance inst_lo + i; first_w(i) = its first weight.
            auto sweep = [&](const int64_t *offs, int n_offs, auto first_w) {
                for (int64_t p = t0 + (int64_t)threadIdx.x * 4; p < t1; p += (int64_t)kPfThreads * 4) {
                    uint32_t w[4];
                    const bool full = p + 4 <= total;
                    if (full && wide_ok) {
                        const uint4 v = *reinterpret_cast<const uint4 *>(chunk_w + p);
                        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) w[e] = (p + e < total) ? chunk_w[p + e] : 0u;
                    }
                    int li = last_le<int64_t>(offs, n_offs, p);
                    uint32_t packed = 0;
                    int64_t miss_inst = -1, miss_pos = 0;      // first mismatch seen by this thread, per instance
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (p + e >= total) break;
                        int64_t nxt = offs[li + 1];
                        while (p + e >= nxt) { ++li; nxt = offs[li + 1]; }
                        const int64_t b = offs[li];
                        const uint32_t w0 = first_w(li, b);
                        const int64_t i = p + e - b;
                        const uint32_t r = nmask >= 0 ? ((uint32_t)i & (uint32_t)nmask) : (uint32_t)((uint64_t)i % (uint64_t)N);
                        packed |= r << (8 * e);
                        if (w[e] != w0 && miss_inst != inst_lo + li) {
                            if (miss_inst >= 0 && run_end[miss_inst * N] > miss_pos) atomicMin((long long *)&run_end[miss_inst * N], (long long)miss_pos);
                            miss_inst = inst_lo + li; miss_pos = i;
                        }
                    }
                    // most positions behind the run's end find a smaller value already there and skip the atomic
                    if (miss_inst >= 0 && run_end[miss_inst * N] > miss_pos) atomicMin((long long *)&run_end[miss_inst * N], (long long)miss_pos);
                    if (full && wide_ok) {
                        *reinterpret_cast<uint32_t *>(rail + p) = packed;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) if (p + e < total) rail[p + e] = (uint8_t)(packed >> (8 * e));
                    }
                }
            };
            if (staged) sweep(s_off, cnt, [&](int li, int64_t) { return s_w0[li]; });
            else sweep(chunk_off + inst_lo, n_inst - inst_lo, [&](int, int64_t b) { return chunk_w[b]; });
        }
    }
}

// ================================================================================ packed shape
// value held by lane T of the caller's GW-lane group
template <int GW, int T>
__device__ __forceinline__ unsigned group_bcast(unsigned v)
{
    if constexpr (GW == 64) return (unsigned)__builtin_amdgcn_readlane((int)v, T);
    else return (unsigned)__builtin_amdgcn_ds_swizzle((int)v, ((0x1F & ~(GW - 1)) | (T << 5)));   // lane = (lane & ~(GW-1)) | T
}

// Broadcast CNT weights of a period (chunks BASE .. BASE + CNT) to their whole group, already shifted into key
// position, before their chain starts, so that the exchange latency is paid once and not once per chunk.
template <int GW, int STEP, int BASE, int CNT, int T>
__device__ __forceinline__ void bcast_steps(const unsigned (&wv)[STEP / GW], unsigned (&bc)[CNT])
{
    if constexpr (T < CNT) {
        bc[T] = group_bcast<GW, (BASE + T) % GW>(wv[(BASE + T) / GW]) << GroupBits<GW>::S;
        bcast_steps<GW, STEP, BASE, CNT, T + 1>(wv, bc);
    }
}

template <int GW, int STEP, int BASE, int CNT, int T>
__device__ __forceinline__ void fast_steps(unsigned &key, const unsigned (&bc)[CNT], unsigned (&won)[STEP / GW], unsigned q)
{
    // chunk BASE + T of the period; the serial chain is: group min (log2 GW exchanges), compare, select
    if constexpr (T < CNT) {
        unsigned bumped = key + bc[T];              // off the chain: does not need the minimum
        asm volatile("" : "+v"(bumped));           // (stops the rewrite into key + select(w, 0), which puts the add on the chain)
        const unsigned m = group_min_u32<GW>(key);
        won[(BASE + T) / GW] = (q == (unsigned)((BASE + T) % GW)) ? m : won[(BASE + T) / GW];
        key = (key == m) ? bumped : key;
        fast_steps<GW, STEP, BASE, CNT, T + 1>(key, bc, won, q);
    }
}

// the period in blocks of CNT chunks: CNT broadcast weights are held at a time
template <int GW, int STEP, int CNT, int BASE>
__device__ __forceinline__ void fast_period(unsigned &key, const unsigned (&wv)[STEP / GW], unsigned (&won)[STEP / GW], unsigned q)
{
    if constexpr (BASE < STEP) {
        unsigned bc[CNT];
        bcast_steps<GW, STEP, BASE, CNT, 0>(wv, bc);
        fast_steps<GW, STEP, BASE, CNT, 0>(key, bc, won, q);
        fast_period<GW, STEP, CNT, BASE + CNT>(key, wv, won, q);
    }
}

// Weights beyond the packing limit: exact 64-bit loads, (load, rail) reductions.  Rare, so kept small: the chunks
// of one register are walked by a loop, the weight fetched from the lane that the loop counter names.
template <int GW, int STEP>
__device__ __forceinline__ void exact_steps(unsigned long long &load, const unsigned (&wv)[STEP / GW], unsigned (&won)[STEP / GW],
                                            unsigned q)
{
#pragma unroll
    for (int r = 0; r < STEP / GW; ++r) {
#pragma unroll 1
        for (int j = 0; j < GW; ++j) {
            const unsigned w = (unsigned)__shfl((int)wv[r], j, GW);
            const unsigned js = group_argmin_u64<GW>(load, q);
            load += (q == js) ? (unsigned long long)w : 0ull;
            won[r] = (q == (unsigned)j) ? js : won[r];
        }
    }
}

// One instance on this wavefront, one chunk per lane and period (the loop is lpt_wide_body in lpt_core.h).
template <int GW, bool RUNS>
__device__ __forceinline__ void wide_instance(int inst, const int64_t *__restrict__ chunk_off, const uint32_t *__restrict__ chunk_w,
                                              int n_inst, int N, uint8_t *__restrict__ rail, int64_t *__restrict__ S_out)
{
    int64_t beg = chunk_off[inst];
    int64_t len = chunk_off[inst + 1] - beg;
    unsigned long long base = 0;
    if (RUNS && len > 0) {
        // skip the leading run (already assigned round robin): start behind it with equal loads
        const unsigned w0 = chunk_w[beg];
        int64_t r0 = S_out[(int64_t)inst * N];
        r0 = r0 < len ? r0 : len;
        if (w0 != 0u && w0 <= WideLimit<GW>::value) {
            const int64_t skip = r0 - r0 % N;
            base = (unsigned long long)w0 * (unsigned long long)(skip / N);
            beg += skip; len -= skip;
        }
    }
    if (!RUNS) prioritise_long_chain(len, chunk_off[n_inst] / n_inst);
    lpt_wide_body<GW, RUNS>(chunk_w + beg, rail + beg, len, base, N, S_out + (int64_t)inst * N,
                            reinterpret_cast<const uint32_t *>(chunk_off));
    if (!RUNS) __builtin_amdgcn_s_setprio(0);
}

// QUEUE: the wavefronts of a small resident grid fetch groups of 64/GW instances from a counter, in the order `order` lists the
// instances (longest first): chains of similar length share a wavefront, long chains start first and short ones fill in behind
// them - list scheduling of the instances over the SIMDs.  The first next_group[2] instances of the order (the few far
// longer than the rest, chosen by the order kernel) are taken one per wavefront before that, through the counter
// next_group[1]: alone on a wavefront a chain advances in three quarters of the time it needs as one of 64/GW, and the
// launch lasts as long as its longest chain.  Without QUEUE wavefront g takes instances g*IPW .. g*IPW + IPW - 1.
template <int GW, bool RUNS, bool QUEUE>
__global__ __launch_bounds__(64 * kLptWaves) void lpt_packed_kernel(const int64_t *__restrict__ chunk_off,
                                                                    const uint32_t *__restrict__ chunk_w, int n_inst, int N,
                                                                    uint8_t *__restrict__ rail, int64_t *__restrict__ S_out,
                                                                    int64_t capacity, const uint32_t *__restrict__ order,
                                                                    unsigned *next_group)
{
    constexpr int S = GroupBits<GW>::S;
    constexpr int IPW = 64 / GW;                    // instances per wavefront
    constexpr int STEP = GW <= 4 ? kBatch / 2 : kBatch;   // chunks per instance and period (GW = 4 holds 8 weights per lane and period already)
    constexpr int REGS = STEP / GW;
    // packing limit: inside a period no delta exceeds (STEP + 2) maximal weights, and the largest
    // packed key must stay below the all-ones key of lanes that hold no rail
    constexpr unsigned W_LIMIT = (unsigned)((0xFFFFFFFFu >> S) / (unsigned)(STEP + 2)) - 1u;

    const int lane = threadIdx.x & 63;
    const unsigned q = (unsigned)(lane % GW);
    const int wave = (int)((blockIdx.x * (unsigned)kLptWaves) + (threadIdx.x >> 6));
    if (chunk_off[n_inst] > capacity) {             // more chunks than the record arrays hold: touch none, mark the loads
        const int64_t n = (int64_t)n_inst * N, stride = (int64_t)gridDim.x * blockDim.x;
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) S_out[i] = -1;
        return;
    }
    const int n_groups = (n_inst + IPW - 1) / IPW;
    auto next = [&]() {
        unsigned g = 0;
        if (lane == 0) g = atomicAdd(next_group, 1u);
        return (int)__builtin_amdgcn_readfirstlane((int)g);
    };
    const int64_t mean_len = chunk_off[n_inst] / n_inst;
    if constexpr (QUEUE) {
        const unsigned n_alone = next_group[2];
        while (true) {
            unsigned i = 0;
            if (lane == 0) i = atomicAdd(next_group + 1, 1u);
            i = (unsigned)__builtin_amdgcn_readfirstlane((int)i);
            if (i >= n_alone) break;                // every wavefront gets here: the counter only grows
            wide_instance<GW, RUNS>((int)order[i], chunk_off, chunk_w, n_inst, N, rail, S_out);
        }
    }
    for (int group = QUEUE ? next() : wave; group < n_groups; group = QUEUE ? next() : n_groups) {
    const int slot = group * IPW + lane / GW;
    const bool has_inst = slot < n_inst;
    const int inst = has_inst ? (QUEUE ? (int)order[slot] : slot) : 0;
    const bool has_rail = has_inst && (int)q < N;
    int64_t beg = has_inst ? chunk_off[inst] : 0;
    int64_t len = has_inst ? chunk_off[inst + 1] - beg : 0;
    unsigned long long base = 0;
    if (RUNS && len > 0) {
        // skip the leading run (already assigned round robin): start behind it with equal loads
        const unsigned w0 = chunk_w[beg];
        int64_t r0 = S_out[(int64_t)inst * N];
        r0 = r0 < len ? r0 : len;
        if (w0 != 0u && w0 <= W_LIMIT) {
            const int64_t skip = r0 - r0 % N;
            base = (unsigned long long)w0 * (unsigned long long)(skip / N);
            beg += skip; len -= skip;
        }
    }

    int64_t max_len = len;                          // the wave runs as long as its longest instance
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) { const int64_t o = __shfl_xor(max_len, d); max_len = o > max_len ? o : max_len; }

    if (!RUNS) prioritise_long_chain(max_len, mean_len);

    unsigned key = has_rail ? q : 0xFFFFFFFFu;
    unsigned long long load = has_rail ? 0ull : ~0ull;
    bool exact = false;                             // wave-uniform

    const unsigned per_rank = (unsigned)(STEP / N), extra = (unsigned)(STEP % N);
    unsigned want[REGS];                            // rank that owns each of this lane's chunks of a period
#pragma unroll
    for (int r = 0; r < REGS; ++r) want[r] = (unsigned)(r * GW + q) % (unsigned)N;

    // Weights of period p: lane q of a group holds chunks p*STEP + r*GW + q; past the end weight 0 (changes nothing).
    // The weights of period p + 2 are requested before the chain of period p and taken in behind it, before the
    // rails are stored.  Lanes past the end of their instance load a word that exists (their instance's last
    // weight, or a spare word once the instance is done) instead of skipping the load: a branch around the loads
    // made the compiler wait for everything in flight - the request just issued and the stores of the period
    // before - in front of every chain.  Positions are compared as 32-bit distances to the end of the instance
    // (`left`, capped far above a period) and addressed from one pointer per period.
    const uint32_t *const spare = reinterpret_cast<const uint32_t *>(chunk_off);
    unsigned in_period[REGS];                       // position of this lane's chunk r inside a period
#pragma unroll
    for (int r = 0; r < REGS; ++r) in_period[r] = (unsigned)(r * GW) + q;
    auto left_at = [&](int64_t i0) {                // chunks of the instance from position i0 on, capped at 2^30
        const int64_t d = len - i0;
        return (unsigned)(d < 0 ? 0 : d > (int64_t)(1 << 30) ? (int64_t)(1 << 30) : d);
    };
    auto request = [&](int64_t i0, unsigned left, unsigned (&wv)[REGS]) {
        const uint32_t *from = left ? chunk_w + beg + i0 : spare;
        const unsigned last = left ? left - 1u : 0u;
#pragma unroll
        for (int r = 0; r < REGS; ++r) wv[r] = from[in_period[r] < last ? in_period[r] : last];
    };
    auto take_in = [&](unsigned left, unsigned (&wv)[REGS]) {
#pragma unroll
        for (int r = 0; r < REGS; ++r) {
            asm volatile("" : "+v"(wv[r]) : : "memory");    // nothing below (the stores least of all) moves above the wait
            wv[r] = in_period[r] < left ? wv[r] : 0u;
        }
    };
    unsigned wv_cur[REGS], wv_nxt[REGS];
    unsigned left = left_at(0), left_nxt = left_at(STEP);   // of the period in hand and of the one after it
    request(0, left, wv_cur);
    request(STEP, left_nxt, wv_nxt);
    take_in(left, wv_cur);
    take_in(left_nxt, wv_nxt);

    for (int64_t i0 = 0; i0 < max_len; i0 += STEP) {
        unsigned wv_far[REGS], won[REGS];
        const unsigned left_far = left_at(i0 + 2 * STEP);
        request(i0 + 2 * STEP, left_far, wv_far);
#pragma unroll
        for (int r = 0; r < REGS; ++r) won[r] = 0;
        if (!exact) {
            unsigned big = 0;
#pragma unroll
            for (int r = 0; r < REGS; ++r) big |= (wv_cur[r] > W_LIMIT) ? 1u : 0u;
            if (__ballot(big != 0) != 0ull) {       // leave the packed representation for good
                exact = true;
                if (has_rail) load = base + (unsigned long long)(key >> S);
            }
        }
        bool closed = false;                        // wave-uniform
        unsigned w0 = 0;
        if (RUNS && !exact) {
            const bool done = left == 0u;           // this group's instance is already finished
            w0 = group_bcast<GW, 0>(wv_cur[0]);
            bool same = true;
#pragma unroll
            for (int r = 0; r < REGS; ++r) same = same && (wv_cur[r] == w0);
            const unsigned dmin = group_min_u32<GW>(key) >> S;
            const unsigned dmax = group_max_u32<GW>(has_rail ? (key >> S) : 0u);
            const bool ok = done || (same && w0 != 0u && left >= (unsigned)STEP && (dmax - dmin) < w0);
            closed = __ballot(!ok) == 0ull;
            if (done) w0 = 0;
        }
        if (closed) {
            const unsigned rank = closed_period<GW>(key, has_rail, w0, per_rank, extra);
#pragma unroll
            for (int r = 0; r < REGS; ++r) won[r] = rail_of_rank<GW>(rank, q, want[r]);
        } else if (!exact) {
            fast_period<GW, STEP, (STEP > 32 ? 32 : STEP), 0>(key, wv_cur, won, q);
#pragma unroll
            for (int r = 0; r < REGS; ++r) won[r] &= (unsigned)(GW - 1);
        } else {
            exact_steps<GW, STEP>(load, wv_cur, won, q);
        }
        if (!exact) {
            // advance the base to the current minimum so deltas stay below the packing limit
            const unsigned adv = group_min_u32<GW>(key) >> S;
            if (has_rail) { key -= adv << S; base += adv; }
        }
        take_in(left_far, wv_far);
        uint8_t *const to = rail + beg + i0 + q;
#pragma unroll
        for (int r = 0; r < REGS; ++r)
            if (in_period[r] < left) to[r * GW] = (uint8_t)won[r];
#pragma unroll
        for (int r = 0; r < REGS; ++r) { wv_cur[r] = wv_nxt[r]; wv_nxt[r] = wv_far[r]; }
        left = left_nxt; left_nxt = left_far;
    }
    if (has_rail) S_out[(int64_t)inst * N + q] = (int64_t)(exact ? load : base + (unsigned long long)(key >> S));
    if (!RUNS) __builtin_amdgcn_s_setprio(0);
    }
}

// ================================================================================ rows shape (N <= 16)
// Four instances per wavefront, one per row of 16 lanes, each in the sorted form of lpt_core.h: a row's first N lanes hold
// its instance's keys in ascending order (as complements), the greedy step is "head plus weight, re-inserted by a median
// of three", five instructions for the four instances (weight to its row through DPP, subtract from the head through DPP,
// neighbour through DPP, v_med3_u32, and a DPP row shift that files the decision) with two of them on the chain - against
// eight and an LDS swizzle with five on the chain for eight instances in the packed shape.  Per instance that is a tenth
// more issue slots and less than half the latency: the shape for batches that the wide shape would crowd and that leave the
// packed one short of wavefronts.  Weights of a period sit four per lane (chunk c*16 + r in register c of lane r), as in
// the packed shape with groups of 16, whose exact 64-bit path (exact_steps) and queue this kernel shares.
template <int T>
__device__ __forceinline__ unsigned row_lane(unsigned v)           // lane T of this lane's row
{
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x150 + T, 0xF, 0xF, true);
}
__device__ __forceinline__ unsigned row_shift_in(unsigned reg, unsigned v)   // every lane takes the next lane's reg, the row's last lane v
{
    return (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)reg, 0x101, 0xF, 0xF, false);
}
// the 16 steps whose weights (shifted past the rail bits) sit in wS, one per lane of the row
template <int T>
__device__ __forceinline__ void rows_steps(unsigned &t, unsigned &won, unsigned wS)
{
    if constexpr (T < 16) {
        const unsigned w = row_lane<T>(wS);
        const unsigned y = list_head<true>(t) - w;
        const unsigned nb = list_next<true>(t);
        won = row_shift_in(won, y);
        t = umed3(t, nb, y);
        rows_steps<T + 1>(t, won, wS);
    }
}

template <int GW, bool RUNS, bool QUEUE>
__global__ __launch_bounds__(64 * kLptWaves) void lpt_rows_kernel(const int64_t *__restrict__ chunk_off,
                                                                  const uint32_t *__restrict__ chunk_w, int n_inst, int N,
                                                                  uint8_t *__restrict__ rail, int64_t *__restrict__ S_out,
                                                                  int64_t capacity, const uint32_t *__restrict__ order,
                                                                  unsigned *next_group)
{
    static_assert(GW <= 16, "an instance's rails fit a row of 16 lanes");
    constexpr int S = GroupBits<GW>::S;             // rail bits of a key (the packing limit follows from them)
    constexpr unsigned MASK = (unsigned)GW - 1u;
    constexpr int LW = 16, IPW = 64 / LW, STEP = kBatch, REGS = STEP / LW;
    constexpr unsigned W_LIMIT = (unsigned)((0xFFFFFFFFu >> S) / (unsigned)(STEP + 2)) - 1u;

    const int lane = threadIdx.x & 63;
    const unsigned r = (unsigned)lane & 15u;
    const int row_base = lane & ~15;
    const int wave = (int)((blockIdx.x * (unsigned)kLptWaves) + (threadIdx.x >> 6));
    if (chunk_off[n_inst] > capacity) {             // more chunks than the record arrays hold: touch none, mark the loads
        const int64_t n = (int64_t)n_inst * N, stride = (int64_t)gridDim.x * blockDim.x;
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) S_out[i] = -1;
        return;
    }
    const int n_groups = (n_inst + IPW - 1) / IPW;
    auto next = [&]() {
        unsigned g = 0;
        if (lane == 0) g = atomicAdd(next_group, 1u);
        return (int)__builtin_amdgcn_readfirstlane((int)g);
    };
    const int64_t mean_len = chunk_off[n_inst] / n_inst;
    if constexpr (QUEUE) {
        const unsigned n_alone = next_group[2];
        while (true) {
            unsigned i = 0;
            if (lane == 0) i = atomicAdd(next_group + 1, 1u);
            i = (unsigned)__builtin_amdgcn_readfirstlane((int)i);
            if (i >= n_alone) break;                // every wavefront gets here: the counter only grows
            wide_instance<GW, RUNS>((int)order[i], chunk_off, chunk_w, n_inst, N, rail, S_out);
        }
    }
    const unsigned per_rank = (unsigned)(STEP / N), extra = (unsigned)(STEP % N);
    const int after_closed = row_base | (int)((r + extra) % (unsigned)N);       // lane whose entry moves here when a list rotates by `extra`
    int place_of_chunk[REGS];                                                   // lane whose entry names the rail of chunk c*16 + r of a closed period
#pragma unroll
    for (int c = 0; c < REGS; ++c) place_of_chunk[c] = row_base | (int)(((unsigned)(c * LW) + r) % (unsigned)N);

    for (int group = QUEUE ? next() : wave; group < n_groups; group = QUEUE ? next() : n_groups) {
    const int slot = group * IPW + lane / LW;
    const bool has_inst = slot < n_inst;
    const int inst = has_inst ? (QUEUE ? (int)order[slot] : slot) : 0;
    const bool in_list = has_inst && (int)r < N;
    int64_t beg = has_inst ? chunk_off[inst] : 0;
    int64_t len = has_inst ? chunk_off[inst + 1] - beg : 0;
    unsigned long long base = 0;
    if (RUNS && len > 0) {
        // skip the leading run (already assigned round robin): start behind it with equal loads
        const unsigned w0 = chunk_w[beg];
        int64_t r0 = S_out[(int64_t)inst * N];
        r0 = r0 < len ? r0 : len;
        if (w0 != 0u && w0 <= W_LIMIT) {
            const int64_t skip = r0 - r0 % N;
            base = (unsigned long long)w0 * (unsigned long long)(skip / N);
            beg += skip; len -= skip;
        }
    }
    int64_t max_len = len;                          // the wave runs as long as its longest instance
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) { const int64_t o = __shfl_xor(max_len, d); max_len = o > max_len ? o : max_len; }
    if (!RUNS) prioritise_long_chain(max_len, mean_len);

    unsigned t = in_list ? ~r : 0u;                 // all deltas 0: ascending rail index
    unsigned long long load = in_list ? 0ull : ~0ull;   // exact path: loads by rail, lane r of the row
    bool exact = false;                             // wave-uniform

    // weights: as in the packed shape (requests two periods ahead, no branch around the loads)
    const uint32_t *const spare = reinterpret_cast<const uint32_t *>(chunk_off);
    unsigned in_period[REGS];
#pragma unroll
    for (int c = 0; c < REGS; ++c) in_period[c] = (unsigned)(c * LW) + r;
    auto left_at = [&](int64_t i0) {
        const int64_t d = len - i0;
        return (unsigned)(d < 0 ? 0 : d > (int64_t)(1 << 30) ? (int64_t)(1 << 30) : d);
    };
    auto request = [&](int64_t i0, unsigned left, unsigned (&wv)[REGS]) {
        const uint32_t *from = left ? chunk_w + beg + i0 : spare;
        const unsigned last = left ? left - 1u : 0u;
#pragma unroll
        for (int c = 0; c < REGS; ++c) wv[c] = from[in_period[c] < last ? in_period[c] : last];
    };
    auto take_in = [&](unsigned left, unsigned (&wv)[REGS]) {
#pragma unroll
        for (int c = 0; c < REGS; ++c) {
            asm volatile("" : "+v"(wv[c]) : : "memory");    // nothing below (the stores least of all) moves above the wait
            wv[c] = in_period[c] < left ? wv[c] : 0u;
        }
    };
    unsigned wv_cur[REGS], wv_nxt[REGS];
    unsigned left = left_at(0), left_nxt = left_at(STEP);
    request(0, left, wv_cur);
    request(STEP, left_nxt, wv_nxt);
    take_in(left, wv_cur);
    take_in(left_nxt, wv_nxt);

    for (int64_t i0 = 0; i0 < max_len; i0 += STEP) {
        unsigned wv_far[REGS], won[REGS];
        const unsigned left_far = left_at(i0 + 2 * STEP);
        request(i0 + 2 * STEP, left_far, wv_far);
#pragma unroll
        for (int c = 0; c < REGS; ++c) won[c] = 0;
        if (!exact) {
            unsigned big = 0;
#pragma unroll
            for (int c = 0; c < REGS; ++c) big |= (wv_cur[c] > W_LIMIT) ? 1u : 0u;
            if (__ballot(big != 0) != 0ull) {       // leave the packed keys for good: lane r takes the entry of rail r
                exact = true;
                for (int place = 0; place < N; ++place) {
                    const unsigned key = ~(unsigned)__shfl((int)t, row_base | place);
                    if (in_list && (key & MASK) == r) load = base + (unsigned long long)(key >> S);
                }
            }
        }
        bool closed = false;                        // wave-uniform
        unsigned w0 = 0;
        if (RUNS && !exact) {
            const bool done = left == 0u;           // this row's instance is already finished
            w0 = row_lane<0>(wv_cur[0]);
            bool same = true;
#pragma unroll
            for (int c = 0; c < REGS; ++c) same = same && (wv_cur[c] == w0);
            const unsigned dmin = (~list_head<true>(t)) >> S;
            const unsigned dmax = (~(unsigned)__shfl((int)t, row_base | (N - 1))) >> S;
            const bool ok = done || (same && w0 != 0u && left >= (unsigned)STEP && (dmax - dmin) < w0);
            closed = __ballot(!ok) == 0ull;
            if (closed && !done) {
                // equal weights from loads within one weight of each other: the list is visited front to back, round after
                // round, and afterwards the places that took one chunk fewer come first: the list rotated by STEP mod N
#pragma unroll
                for (int c = 0; c < REGS; ++c) won[c] = (~(unsigned)__shfl((int)t, place_of_chunk[c])) & MASK;
                const unsigned grown = t - ((w0 * (per_rank + (r < extra ? 1u : 0u))) << S);
                const unsigned moved = (unsigned)__shfl((int)grown, after_closed);
                t = in_list ? moved : 0u;
            }
        }
        if (closed) {
        } else if (!exact) {
#pragma unroll
            for (int c = 0; c < REGS; ++c) {
                rows_steps<0>(t, won[c], wv_cur[c] << S);
                won[c] = ~won[c] & MASK;
            }
        } else {
            exact_steps<LW, STEP>(load, wv_cur, won, r);
        }
        if (!exact) {
            // the emptiest rail's delta moves into the base, so deltas stay below the packing limit
            const unsigned adv = (~list_head<true>(t)) >> S;
            if (in_list) { t += adv << S; base += adv; }
        }
        take_in(left_far, wv_far);
        uint8_t *const to = rail + beg + i0 + r;
#pragma unroll
        for (int c = 0; c < REGS; ++c)
            if (in_period[c] < left) to[c * LW] = (uint8_t)won[c];
#pragma unroll
        for (int c = 0; c < REGS; ++c) { wv_cur[c] = wv_nxt[c]; wv_nxt[c] = wv_far[c]; }
        left = left_nxt; left_nxt = left_far;
    }
    if (in_list) {
        if (exact) {
            S_out[(int64_t)inst * N + r] = (int64_t)load;
        } else {
            const unsigned key = ~t;
            S_out[(int64_t)inst * N + (key & MASK)] = (int64_t)(base + (unsigned long long)(key >> S));
        }
    }
    if (!RUNS) __builtin_amdgcn_s_setprio(0);
    }
}

// Instances in descending order of chain length, to within the resolution of 512 buckets (a sixteenth of the length): counting
// sort by one workgroup.  RUNS: S[inst*N] holds the length of the instance's leading run, which the serial kernel skips.
// Also sets the counters of the queue: next_group[0] = first group the packed wavefronts take, [1] = 0 (next instance to run
// alone), [2] = how many of the longest run alone: those at least half as long again as the mean and longer than a
// 24 576th of all chunks (below that the packed chains are done before the launch's issue slots are), a whole number of
// groups, at most 64.
constexpr int kOrdBuckets = 512;
__device__ __forceinline__ int order_bucket(uint64_t len)
{
    if (len < 32) return (int)len;                                      // exact below 32
    if (len >> 32) return kOrdBuckets - 1;
    const int e = 31 - __clz((int)(uint32_t)len);                       // 5 .. 31
    return 32 + (e - 5) * 16 + (int)((len >> (e - 4)) & 15u);           // 16 steps per power of two: 32 .. 463
}
template <bool RUNS>
__global__ __launch_bounds__(1024) void lpt_order_kernel(const int64_t *__restrict__ chunk_off, const int64_t *__restrict__ S, int n_inst, int N,
                                                         int ipw, uint32_t *__restrict__ order, unsigned *next_group)
{
    __shared__ unsigned hist[kOrdBuckets];
    __shared__ unsigned long long sum_len;
    for (int i = threadIdx.x; i < kOrdBuckets; i += 1024) hist[i] = 0;
    if (threadIdx.x == 0) sum_len = 0;
    __syncthreads();
    auto length = [&](int i) {
        int64_t len = chunk_off[i + 1] - chunk_off[i];
        if (RUNS) { int64_t r0 = S[(int64_t)i * N]; r0 = r0 < len ? r0 : len; len -= r0 - r0 % N; }
        return (uint64_t)(len < 0 ? 0 : len);
    };
    unsigned long long mine = 0;
    for (int i = threadIdx.x; i < n_inst; i += 1024) { const uint64_t len = length(i); mine += len; atomicAdd(&hist[order_bucket(len)], 1u); }
    for (int d = 32; d >= 1; d >>= 1) mine += __shfl_xor(mine, d);
    if ((threadIdx.x & 63) == 0) atomicAdd(&sum_len, mine);
    __syncthreads();
    if (threadIdx.x < 64) {                                             // exclusive scan from the longest bucket down: 8 buckets per lane
        const int hi = kOrdBuckets - 1 - (int)threadIdx.x * 8;
        unsigned v[8], sum = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) { v[j] = hist[hi - j]; sum += v[j]; }
        unsigned total;
        unsigned ex = wave_exscan(sum, total);
#pragma unroll
        for (int j = 0; j < 8; ++j) { hist[hi - j] = ex; ex += v[j]; }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        // hist[b] = instances in buckets above b = where bucket b starts in the order: everything before the bucket of the
        // threshold is longer than the threshold
        const uint64_t total = sum_len, mean = total / (uint64_t)n_inst;
        uint64_t thresh = mean + mean / 2;
        if (thresh < total / 24576) thresh = total / 24576;
        unsigned alone = thresh > 0 ? hist[order_bucket(thresh)] : 0u;
        alone = alone > 64u ? 64u : alone;
        alone -= alone % (unsigned)ipw;
        next_group[0] = alone / (unsigned)ipw;
        next_group[1] = 0;
        next_group[2] = alone;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n_inst; i += 1024) order[atomicAdd(&hist[order_bucket(length(i))], 1u)] = (uint32_t)i;
}

// ================================================================================ wide shape (loop in lpt_core.h)
template <int GW, bool RUNS>
__global__ __launch_bounds__(64 * kLptWaves) void lpt_wide_kernel(const int64_t *__restrict__ chunk_off,
                                                                  const uint32_t *__restrict__ chunk_w, int n_inst, int N,
                                                                  uint8_t *__restrict__ rail, int64_t *__restrict__ S_out,
                                                                  int64_t capacity)
{
    const int inst = (int)((blockIdx.x * (unsigned)kLptWaves) + (threadIdx.x >> 6));
    if (inst >= n_inst) return;                     // whole wavefront leaves; nothing below synchronises across waves
    if (chunk_off[n_inst] > capacity) {             // more chunks than the record arrays hold: touch none, mark the loads
        if ((int)(threadIdx.x & 63) < N) S_out[(int64_t)inst * N + (threadIdx.x & 63)] = -1;
        return;
    }
    wide_instance<GW, RUNS>(inst, chunk_off, chunk_w, n_inst, N, rail, S_out);
}


// serial kernels only: every instance's S_out[inst*N] must hold the length of its leading run (or less)
// workspace of the serial kernels: the instance order (one word per instance) and, 256 bytes behind it, the group counter
static size_t lpt_ws_bytes(int64_t n_inst) { return align_up(sizeof(uint32_t) * (size_t)n_inst, 256) + 256; }

template <int GW, bool RUNS>
static int launch_lpt_serial(const int64_t *chunk_off, const uint32_t *chunk_w, int64_t n_inst, int N, uint8_t *rail,
                             int64_t *S, int64_t capacity, void *ws, hipStream_t st)
{
    constexpr int IPW = 64 / GW;
    // Three shapes (ns per greedy step and instance-carrying wavefront, measured on batches of equal chains, N = 4, 8, 16):
    //   wide   one instance per wavefront:      16 alone on a SIMD, 25 / 35 / 46 with two / three / four wavefronts on it
    //   rows   four per wavefront (N <= 16):    17-20 up to one wavefront per SIMD, 26 with two, 46 with four
    //   packed 64/GW per wavefront:             34-39 however few, 41 at 16 384 instances (N = 16: 72)
    // so: wide up to one wavefront per SIMD (256 CUs x 4 SIMDs), then rows up to 16 384 instances (always for groups of 16
    // lanes, which pack no denser than rows do), then packed.  N = 32 has no rows shape: wide takes 22 / 28 / 42 / 53 / 75
    // with one to six wavefronts on a SIMD against 64-74 packed, so wide up to five.
    constexpr int64_t kWideMax = GW <= 16 ? 1024 : 5 * 1024;
    constexpr int64_t kRowsMax = GW == 16 ? INT64_MAX : 16384;
    const bool packed = IPW > 1 && n_inst > kWideMax;
    if constexpr (GW <= 16) {
        if (packed && n_inst <= kRowsMax) {
            constexpr int RPW = 4;
            const int64_t waves = (n_inst + RPW - 1) / RPW;
            int64_t blocks = (waves + kLptWaves - 1) / kLptWaves;
            if (ws && !RUNS) {
                // heavy-tailed batches: longest first from a queue, two resident wavefronts per SIMD (four: a fifth slower at 12 288 instances)
                uint32_t *order = static_cast<uint32_t *>(ws);
                unsigned *counter = reinterpret_cast<unsigned *>(static_cast<char *>(ws) + align_up(sizeof(uint32_t) * (size_t)n_inst, 256));
                hipLaunchKernelGGL((lpt_order_kernel<RUNS>), dim3(1), dim3(1024), 0, st, chunk_off, S, (int)n_inst, N, RPW, order, counter);
                if (int rc = launch_status()) return rc;
                const int64_t resident = 256 * 4 * 2 / kLptWaves;
                if (blocks > resident) blocks = resident;
                hipLaunchKernelGGL((lpt_rows_kernel<GW, RUNS, true>), dim3((unsigned)blocks), dim3(64 * kLptWaves), 0, st, chunk_off,
                                   chunk_w, (int)n_inst, N, rail, S, capacity, order, counter);
            } else {
                hipLaunchKernelGGL((lpt_rows_kernel<GW, RUNS, false>), dim3((unsigned)blocks), dim3(64 * kLptWaves), 0, st, chunk_off,
                                   chunk_w, (int)n_inst, N, rail, S, capacity, nullptr, nullptr);
            }
            return launch_status();
        }
    }
    constexpr bool kHasPacked = IPW > 1 && GW != 16;   // groups of 16 lanes always take the rows shape
    if constexpr (kHasPacked) {
    if (packed && ws && !RUNS) {                    // behind the closed forms the chains are a few hundred tails each: nothing to order
        // Three resident wavefronts per SIMD: with the longest chains alone on a wavefront each (and at a raised issue
        // priority) a fourth only slows those chains, which the launch waits for, and with two the SIMDs idle between
        // dependent instructions; fewer wavefronts than groups also leaves every wavefront several groups to even out with.
        uint32_t *order = static_cast<uint32_t *>(ws);
        unsigned *counter = reinterpret_cast<unsigned *>(static_cast<char *>(ws) + align_up(sizeof(uint32_t) * (size_t)n_inst, 256));
        hipLaunchKernelGGL((lpt_order_kernel<RUNS>), dim3(1), dim3(1024), 0, st, chunk_off, S, (int)n_inst, N, IPW, order, counter);
        if (int rc = launch_status()) return rc;
        const int64_t waves = (n_inst + IPW - 1) / IPW;
        int64_t blocks = (waves + kLptWaves - 1) / kLptWaves;
        const int64_t resident = 256 * 4 * 3 / kLptWaves;
        if (blocks > resident) blocks = resident;
        hipLaunchKernelGGL((lpt_packed_kernel<GW, RUNS, true>), dim3((unsigned)blocks), dim3(64 * kLptWaves), 0, st, chunk_off,
                           chunk_w, (int)n_inst, N, rail, S, capacity, order, counter);
        return launch_status();
    } else if (packed) {
        const int64_t waves = (n_inst + IPW - 1) / IPW;
        const int64_t blocks = (waves + kLptWaves - 1) / kLptWaves;
        hipLaunchKernelGGL((lpt_packed_kernel<GW, RUNS, false>), dim3((unsigned)blocks), dim3(64 * kLptWaves), 0, st, chunk_off,
                           chunk_w, (int)n_inst, N, rail, S, capacity, nullptr, nullptr);
        return launch_status();
    }
    }
    const int64_t blocks = (n_inst + kLptWaves - 1) / kLptWaves;
    hipLaunchKernelGGL((lpt_wide_kernel<GW, RUNS>), dim3((unsigned)blocks), dim3(64 * kLptWaves), 0, st, chunk_off,
                       chunk_w, (int)n_inst, N, rail, S, capacity);
    return launch_status();
}

template <int GW, bool RUNS>
static int launch_lpt(const int64_t *chunk_off, const uint32_t *chunk_w, int64_t n_inst, int N, uint8_t *rail,
                      int64_t *S, int64_t capacity, void *ws, hipStream_t st)
{
    if (RUNS) {
        hipLaunchKernelGGL(lpt_prefix_init_kernel, dim3((unsigned)((n_inst + 255) / 256 > 1024 ? 1024 : (n_inst + 255) / 256)), dim3(256),
                           0, st, S, (int)n_inst, N);
        const int wide_ok = (reinterpret_cast<uintptr_t>(chunk_w) % 16 == 0 && reinterpret_cast<uintptr_t>(rail) % 4 == 0) ? 1 : 0;
        hipLaunchKernelGGL(lpt_prefix_kernel, dim3(kPfBlocks), dim3(kPfThreads), 0, st, chunk_off, chunk_w, (int)n_inst, N,
                           is_pow2(N) ? N - 1 : -1, rail, S, wide_ok, capacity);
        if (int rc = launch_status()) return rc;
    }
    return launch_lpt_serial<GW, RUNS>(chunk_off, chunk_w, n_inst, N, rail, S, capacity, ws, st);
}

// for the one-call scheduler, which knows every leading run from stage 3 and has written its rails
int lpt_serial_after_leading_runs(const int64_t *chunk_off, const uint32_t *chunk_w, int64_t n_inst, int N, uint8_t *rail,
                                  int64_t *S, int64_t capacity, hipStream_t st)
{
    if (N <= 4) return launch_lpt_serial<4, true>(chunk_off, chunk_w, n_inst, N, rail, S, capacity, nullptr, st);
    if (N <= 8) return launch_lpt_serial<8, true>(chunk_off, chunk_w, n_inst, N, rail, S, capacity, nullptr, st);
    if (N <= 16) return launch_lpt_serial<16, true>(chunk_off, chunk_w, n_inst, N, rail, S, capacity, nullptr, st);
    if (N <= 32) return launch_lpt_serial<32, true>(chunk_off, chunk_w, n_inst, N, rail, S, capacity, nullptr, st);
    return launch_lpt_serial<64, true>(chunk_off, chunk_w, n_inst, N, rail, S, capacity, nullptr, st);
}

template <bool RUNS>
static int lpt_entry(const int64_t *chunk_off, const uint32_t *chunk_w, int32_t batch, const railsched_topo_t *h_topo,
                     int64_t capacity, uint8_t *rail, int64_t *S, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0 || capacity < 0) return RAILSCHED_ERR_INVALID_ARG;
    const int64_t n_inst = (int64_t)batch * h_topo->nodes;
    if (n_inst > 0x7FFFFFFFll / 64) return RAILSCHED_ERR_UNSUPPORTED;
    if (n_inst == 0) return RAILSCHED_OK;
    if (!chunk_off || !S || (capacity > 0 && (!chunk_w || !rail))) return RAILSCHED_ERR_NULL_PTR;
    if (ws && (ws_bytes < lpt_ws_bytes(n_inst) || reinterpret_cast<uintptr_t>(ws) % 256)) return RAILSCHED_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int N = h_topo->rails;
    if (N <= 4) return launch_lpt<4, RUNS>(chunk_off, chunk_w, n_inst, N, rail, S, capacity, ws, st);
    if (N <= 8) return launch_lpt<8, RUNS>(chunk_off, chunk_w, n_inst, N, rail, S, capacity, ws, st);
    if (N <= 16) return launch_lpt<16, RUNS>(chunk_off, chunk_w, n_inst, N, rail, S, capacity, ws, st);
    if (N <= 32) return launch_lpt<32, RUNS>(chunk_off, chunk_w, n_inst, N, rail, S, capacity, ws, st);
    return launch_lpt<64, RUNS>(chunk_off, chunk_w, n_inst, N, rail, S, capacity, ws, st);
}

}  // namespace rs

extern "C" size_t railsched_lpt_spray_workspace_bytes(int32_t batch, const railsched_topo_t *h_topo)
{
    using namespace rs;
    if (check_topo(h_topo) != RAILSCHED_OK || batch < 0) return 0;
    return lpt_ws_bytes((int64_t)batch * h_topo->nodes);
}

extern "C" int railsched_lpt_spray(const int64_t *chunk_off, const uint32_t *chunk_w, int32_t batch,
                                   const railsched_topo_t *h_topo, int64_t capacity, uint8_t *rail, int64_t *S, void *ws,
                                   size_t ws_bytes, void *stream)
{
    return rs::lpt_entry<true>(chunk_off, chunk_w, batch, h_topo, capacity, rail, S, ws, ws_bytes, stream);
}

extern "C" int railsched_lpt_spray_chunkwise(const int64_t *chunk_off, const uint32_t *chunk_w, int32_t batch,
                                             const railsched_topo_t *h_topo, int64_t capacity, uint8_t *rail, int64_t *S,
                                             void *ws, size_t ws_bytes, void *stream)
{
    return rs::lpt_entry<false>(chunk_off, chunk_w, batch, h_topo, capacity, rail, S, ws, ws_bytes, stream);
}
