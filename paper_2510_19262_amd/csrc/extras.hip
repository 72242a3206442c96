// Extensions around the five core stages:
//  * railsched_transpose_matrix: traffic of the second all-to-all of an MoE layer (Algorithm 1 step 4:
//    expert outputs return to the token owners), i.e. every traffic matrix transposed;
//  * railsched_assign_policy: the path-selection schemes the paper compares against (Sections 1, 2.2,
//    6.1), reduced to arithmetic on the same chunk records: which rail would each chunk take.
#include "common.h"

namespace rs {

// ------------------------------------------------------------------------------------ transpose
constexpr int kTrTile = 32;

__global__ __launch_bounds__(256) void transpose_kernel(const int64_t *__restrict__ in, int64_t *__restrict__ out, int G, int tiles)
{
    __shared__ int64_t tile[kTrTile][kTrTile + 1];
    const int64_t b = blockIdx.x / ((int64_t)tiles * tiles);
    const int t = (int)(blockIdx.x % ((int64_t)tiles * tiles));
    const int ty = t / tiles, tx = t % tiles;
    const int64_t base = b * (int64_t)G * G;
    const int lx = threadIdx.x % kTrTile, ly = threadIdx.x / kTrTile;       // 32 x 8 threads
    for (int j = ly; j < kTrTile; j += 8) {
        const int r = ty * kTrTile + j, c = tx * kTrTile + lx;
        if (r < G && c < G) tile[j][lx] = in[base + (int64_t)r * G + c];
    }
    __syncthreads();
    for (int j = ly; j < kTrTile; j += 8) {
        const int r = tx * kTrTile + j, c = ty * kTrTile + lx;              // transposed block, rows written contiguously
        if (r < G && c < G) out[base + (int64_t)r * G + c] = tile[lx][j];
    }
}

// ------------------------------------------------------------------------------------ comparison schemes
constexpr int kPolThreads = 256;
constexpr int kPolTile = 8192;      // chunk positions per workgroup iteration
constexpr int kPolStage = 1024;     // instance boundaries staged in LDS per tile
constexpr int kPolSlots = 8;        // instances of a tile whose rail loads are accumulated in LDS
constexpr int kPolBlocks = 2048;

struct PolArgs {
    const int64_t *chunk_off;
    const uint32_t *chunk_w, *chunk_flow;
    uint8_t *rail;
    int64_t *S;
    uint64_t seed;
    int32_t n_inst, N, G, NF, policy;
    int32_t nmask, gshift;          // >= 0 when N / G are powers of two
    int32_t wide_ok;
    int64_t capacity;               // records the per-chunk arrays hold
};

__device__ __forceinline__ uint64_t mix64(uint64_t z)                   // splitmix64 finaliser
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ uint32_t mod_n(const PolArgs &a, uint64_t x)
{
    return a.nmask >= 0 ? (uint32_t)x & (uint32_t)a.nmask : (uint32_t)(x % (uint64_t)a.N);
}

__device__ __forceinline__ uint32_t policy_rail(const PolArgs &a, int64_t inst, int64_t pos_global, int64_t pos_in_inst, uint32_t flow)
{
    switch (a.policy) {
        case 0: return a.gshift >= 0 ? flow >> a.gshift : flow / (uint32_t)a.G;                                  // NIC-direct
        case 1: return mod_n(a, mix64(a.seed + 0x9E3779B97F4A7C15ull * ((uint64_t)inst * (uint64_t)a.NF + flow + 1)));   // flow hash
        case 2: return mod_n(a, mix64(a.seed + 0x9E3779B97F4A7C15ull * ((uint64_t)pos_global + 1)));             // random spray
        default: return mod_n(a, (uint64_t)pos_in_inst);                                                        // round robin
    }
}

// S = 0 before the sums; -1 throughout when there are more chunks than the record arrays hold (the policy kernel
// then touches nothing)
__global__ void policy_init_kernel(PolArgs a, int64_t n)
{
    const int64_t v = a.chunk_off[a.n_inst] > a.capacity ? -1 : 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) a.S[i] = v;
}

// Streaming over all chunk positions, four per thread at multiples of four.  Send loads go to LDS bins
// for the first kPolSlots instances a tile touches (a tile rarely touches more) and from there, or
// directly for the rest, to S with integer atomics (S is zeroed first; integer sums are order-free).
__global__ __launch_bounds__(kPolThreads) void policy_kernel(PolArgs a)
{
    __shared__ int64_t s_off[kPolStage + 1];
    __shared__ unsigned long long bins[kPolSlots][kMaxRails];
    const int64_t total = a.chunk_off[a.n_inst];
    if (total > a.capacity) return;
    for (int64_t t0 = (int64_t)blockIdx.x * kPolTile; t0 < total; t0 += (int64_t)gridDim.x * kPolTile) {
        const int64_t t1 = t0 + kPolTile < total ? t0 + kPolTile : total;
        const int inst_lo = wave_last_le<int64_t>(a.chunk_off, a.n_inst, t0);
        const int inst_hi = wave_last_le<int64_t>(a.chunk_off, a.n_inst, t1 - 1);
        const int cnt = inst_hi - inst_lo + 1;
        const bool staged = cnt <= kPolStage;
        __syncthreads();                                   // previous tile is done with the LDS
        if (staged)
            for (int i = threadIdx.x; i <= cnt; i += kPolThreads) s_off[i] = a.chunk_off[inst_lo + i];
        for (int i = threadIdx.x; i < kPolSlots * kMaxRails; i += kPolThreads) (&bins[0][0])[i] = 0ull;
        __syncthreads();
        // one sweep for instance boundaries staged in LDS and one for boundaries read from memory (through a pointer that
        // may be either, every lookup is a flat load, which waits for all of the wavefront's memory traffic);
        // offs[i] = start of instance inst_lo + i
        auto sweep = [&](const int64_t *offs, int n_offs) {
            for (int64_t p = t0 + (int64_t)threadIdx.x * 4; p < t1; p += (int64_t)kPolThreads * 4) {
                uint32_t w[4], fl[4];
                const bool full = p + 4 <= total;
                if (full && a.wide_ok) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(a.chunk_w + p);
                    const uint4 f = *reinterpret_cast<const uint4 *>(a.chunk_flow + p);
                    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
                    fl[0] = f.x; fl[1] = f.y; fl[2] = f.z; fl[3] = f.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        w[e] = (p + e < total) ? a.chunk_w[p + e] : 0u;
                        fl[e] = (p + e < total) ? a.chunk_flow[p + e] : 0u;
                    }
                }
                int li = last_le<int64_t>(offs, n_offs, p);
                uint32_t packed = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (p + e >= total) break;
                    int64_t nxt = offs[li + 1];
                    while (p + e >= nxt) { ++li; nxt = offs[li + 1]; }
                    const int64_t b = offs[li];
                    const uint32_t r = policy_rail(a, inst_lo + li, p + e, p + e - b, fl[e]);
                    packed |= r << (8 * e);
                    if (r < (uint32_t)a.N) {
                        if (li < kPolSlots) atomicAdd(&bins[li][r], (unsigned long long)w[e]);
                        else atomicAdd(reinterpret_cast<unsigned long long *>(a.S + (int64_t)(inst_lo + li) * a.N + r), (unsigned long long)w[e]);
                    }
                }
                if (full && a.wide_ok) {
                    *reinterpret_cast<uint32_t *>(a.rail + p) = packed;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) if (p + e < total) a.rail[p + e] = (uint8_t)(packed >> (8 * e));
                }
            }
        };
        if (staged) sweep(s_off, cnt);
        else sweep(a.chunk_off + inst_lo, a.n_inst - inst_lo);
        __syncthreads();
        for (int i = threadIdx.x; i < kPolSlots * a.N; i += kPolThreads) {
            const int li = i / a.N, r = i % a.N;
            const unsigned long long v = bins[li][r];
            if (v && li < cnt) atomicAdd(reinterpret_cast<unsigned long long *>(a.S + (int64_t)(inst_lo + li) * a.N + r), v);
        }
    }
}

// ------------------------------------------------------------------------------------ port round robin
// Algorithm 2 step 4.  port[i] = (how many earlier chunks of the same instance went to the same rail) mod P.
// Instances are cut into tiles of kPortTile chunks; (1) tile offsets per instance, (2) per-tile per-rail
// counts, (3) per instance an exclusive scan of the counts over its tiles, (4) per tile the running
// counts: one wavefront walks the tile 64 chunks at a time, lanes with the same rail find each other by
// ballot matching, rank = running count + number of lower lanes with that rail.
constexpr int kPortTile = 4096;
constexpr int kPortWaves = 4;
constexpr int kPortBlocks = 2048;

struct PortArgs {
    const int64_t *chunk_off;
    const uint8_t *rail;
    uint8_t *port;
    int64_t *tile_off;          // [n_inst + 1]
    uint32_t *cnt;              // [tiles][N]: counts, then exclusive prefixes inside the instance
    int64_t max_tiles;
    int64_t capacity;           // records rail and port hold
    int32_t n_inst, N, P, pmask, rail_bits;
};

__global__ __launch_bounds__(1024) void port_tiles_kernel(PortArgs a)
{
    __shared__ int64_t sh[1024];
    __shared__ int64_t carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < a.n_inst; base += 1024) {
        const int i = base + tid;
        const int64_t v = i < a.n_inst ? (a.chunk_off[i + 1] - a.chunk_off[i] + kPortTile - 1) / kPortTile : 0;
        sh[tid] = v;
        __syncthreads();
        for (int d = 1; d < 1024; d <<= 1) {
            const int64_t x = tid >= d ? sh[tid - d] : 0;
            __syncthreads();
            sh[tid] += x;
            __syncthreads();
        }
        if (i < a.n_inst) a.tile_off[i] = carry + sh[tid] - v;
        __syncthreads();
        if (tid == 1023) carry += sh[1023];
        __syncthreads();
    }
    if (tid == 0) a.tile_off[a.n_inst] = carry;
}

template <bool ASSIGN>
__global__ __launch_bounds__(64 * kPortWaves) void port_tile_kernel(PortArgs a)
{
    __shared__ unsigned run[kPortWaves][kMaxRails];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const unsigned long long lt = (1ull << lane) - 1ull;
    if (a.chunk_off[a.n_inst] > a.capacity) return;                 // more chunks than rail and port hold: touch neither
    int64_t n_tiles = a.tile_off[a.n_inst];
    if (n_tiles > a.max_tiles) n_tiles = a.max_tiles;               // workspace sized for fewer chunks: never write past it
    unsigned *mine = run[wv];
    for (int64_t u = (int64_t)blockIdx.x * kPortWaves + wv; u < n_tiles; u += (int64_t)gridDim.x * kPortWaves) {
        const int inst = wave_last_le<int64_t>(a.tile_off, a.n_inst, u);
        const int64_t beg = a.chunk_off[inst] + (u - a.tile_off[inst]) * kPortTile;
        const int64_t end = (beg + kPortTile < a.chunk_off[inst + 1]) ? beg + kPortTile : a.chunk_off[inst + 1];
        uint32_t *c = a.cnt + u * a.N;
        if (lane < a.N) mine[lane] = ASSIGN ? c[lane] : 0u;
        __builtin_amdgcn_wave_barrier();
        for (int64_t i0 = beg; i0 < end; i0 += 64) {
            const int64_t i = i0 + lane;
            const bool act = i < end;
            const unsigned r = act ? a.rail[i] : 0u;
            const bool ok = act && r < (unsigned)a.N;
            if (!ASSIGN) {
                if (ok) atomicAdd(&mine[r], 1u);
            } else {
                unsigned long long peers = __ballot(ok);
                for (int bit = 0; bit < a.rail_bits; ++bit) {
                    const bool one = (r >> bit) & 1u;
                    const unsigned long long bm = __ballot(ok && one);
                    peers &= one ? bm : ~bm;
                }
                const unsigned base = ok ? mine[r] : 0u;
                const unsigned rank = base + (unsigned)__popcll(peers & lt);
                if (act) a.port[i] = ok ? (uint8_t)(a.pmask >= 0 ? (rank & (unsigned)a.pmask) : (rank % (unsigned)a.P)) : (uint8_t)0;
                __builtin_amdgcn_wave_barrier();
                if (ok && (peers >> lane) == 1ull) mine[r] = base + (unsigned)__popcll(peers);   // highest lane of the peer set
                __builtin_amdgcn_wave_barrier();
            }
        }
        if (!ASSIGN) {
            __builtin_amdgcn_wave_barrier();
            if (lane < a.N) c[lane] = mine[lane];
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// exclusive scan of the per-tile counts over the tiles of one instance; lane = rail
__global__ __launch_bounds__(64) void port_scan_kernel(PortArgs a)
{
    const int inst = blockIdx.x, lane = threadIdx.x;
    int64_t t0 = a.tile_off[inst], t1 = a.tile_off[inst + 1];
    if (t1 > a.max_tiles) t1 = a.max_tiles;
    if (lane >= a.N) return;
    unsigned running = 0;
    for (int64_t t = t0; t < t1; ++t) {
        const unsigned v = a.cnt[t * a.N + lane];
        a.cnt[t * a.N + lane] = running;
        running += v;
    }
}

static void port_ws_layout(int64_t n_inst, int64_t max_tiles, int N, size_t off[3])
{
    size_t o = 0;
    off[0] = o; o += align_up(sizeof(int64_t) * (size_t)(n_inst + 1), 256);
    off[1] = o; o += align_up(sizeof(uint32_t) * (size_t)max_tiles * (size_t)N, 256);
    off[2] = o;
}

}  // namespace rs

extern "C" int railsched_transpose_matrix(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo, int64_t *D1T,
                                          void *stream)
{
    using namespace rs;
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0) return RAILSCHED_ERR_INVALID_ARG;
    if (batch == 0) return RAILSCHED_OK;
    if (!D1 || !D1T) return RAILSCHED_ERR_NULL_PTR;
    if (D1 == D1T) return RAILSCHED_ERR_INVALID_ARG;     // not in place
    const int G = h_topo->nodes * h_topo->rails;
    const int tiles = (G + kTrTile - 1) / kTrTile;
    const int64_t blocks = (int64_t)batch * tiles * tiles;
    if (blocks > 0x7FFFFFFFll) return RAILSCHED_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), D1, D1T, G, tiles);
    return launch_status();
}

extern "C" int railsched_assign_policy(int32_t policy, uint64_t seed, const int64_t *chunk_off, const uint32_t *chunk_w,
                                       const uint32_t *chunk_flow, int32_t batch, const railsched_topo_t *h_topo,
                                       int64_t capacity, uint8_t *rail, int64_t *S, void *stream)
{
    using namespace rs;
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0 || policy < 0 || policy > 3 || capacity < 0) return RAILSCHED_ERR_INVALID_ARG;
    const int64_t n_inst = (int64_t)batch * h_topo->nodes;
    if (n_inst > 0x7FFFFFFFll / 64) return RAILSCHED_ERR_UNSUPPORTED;
    if (n_inst == 0) return RAILSCHED_OK;
    if (!chunk_off || !S || (capacity > 0 && (!chunk_w || !chunk_flow || !rail))) return RAILSCHED_ERR_NULL_PTR;
    hipStream_t st = static_cast<hipStream_t>(stream);
    PolArgs a;
    a.capacity = capacity;
    a.chunk_off = chunk_off; a.chunk_w = chunk_w; a.chunk_flow = chunk_flow; a.rail = rail; a.S = S; a.seed = seed;
    a.n_inst = (int32_t)n_inst; a.N = h_topo->rails; a.G = h_topo->nodes * h_topo->rails; a.NF = a.N * a.G; a.policy = policy;
    a.nmask = is_pow2(a.N) ? a.N - 1 : -1;
    a.gshift = is_pow2(a.G) ? ilog2(a.G) : -1;
    a.wide_ok = (reinterpret_cast<uintptr_t>(chunk_w) % 16 == 0 && reinterpret_cast<uintptr_t>(chunk_flow) % 16 == 0 &&
                 reinterpret_cast<uintptr_t>(rail) % 4 == 0) ? 1 : 0;
    const int64_t n = n_inst * a.N;
    hipLaunchKernelGGL(policy_init_kernel, dim3((unsigned)((n + 255) / 256 > 1024 ? 1024 : (n + 255) / 256)), dim3(256), 0, st, a, n);
    if (int rc = launch_status()) return rc;
    hipLaunchKernelGGL(policy_kernel, dim3(kPolBlocks), dim3(kPolThreads), 0, st, a);
    return launch_status();
}

extern "C" size_t railsched_port_round_robin_workspace_bytes(int32_t batch, const railsched_topo_t *h_topo, int64_t capacity)
{
    using namespace rs;
    if (check_topo(h_topo) != RAILSCHED_OK || batch < 0 || capacity < 0) return 0;
    const int64_t n_inst = (int64_t)batch * h_topo->nodes;
    size_t off[3];
    port_ws_layout(n_inst, capacity / kPortTile + n_inst + 1, h_topo->rails, off);
    return off[2];
}

extern "C" int railsched_port_round_robin(const int64_t *chunk_off, const uint8_t *rail, int32_t batch,
                                          const railsched_topo_t *h_topo, int32_t ports, int64_t capacity, uint8_t *port,
                                          void *ws, size_t ws_bytes, void *stream)
{
    using namespace rs;
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0 || capacity < 0 || ports < 1) return RAILSCHED_ERR_INVALID_ARG;
    if (ports > 256) return RAILSCHED_ERR_UNSUPPORTED;
    const int64_t n_inst = (int64_t)batch * h_topo->nodes;
    if (n_inst > 0x7FFFFFFFll / 64) return RAILSCHED_ERR_UNSUPPORTED;
    if (n_inst == 0) return RAILSCHED_OK;
    if (!chunk_off || (capacity > 0 && (!rail || !port))) return RAILSCHED_ERR_NULL_PTR;
    const int64_t max_tiles = capacity / kPortTile + n_inst + 1;
    size_t off[3];
    port_ws_layout(n_inst, max_tiles, h_topo->rails, off);
    if (!ws || ws_bytes < off[2] || reinterpret_cast<uintptr_t>(ws) % 256) return RAILSCHED_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    PortArgs a;
    a.chunk_off = chunk_off; a.rail = rail; a.port = port;
    a.tile_off = reinterpret_cast<int64_t *>(static_cast<char *>(ws) + off[0]);
    a.cnt = reinterpret_cast<uint32_t *>(static_cast<char *>(ws) + off[1]);
    a.max_tiles = max_tiles; a.capacity = capacity;
    a.n_inst = (int32_t)n_inst; a.N = h_topo->rails; a.P = ports; a.pmask = is_pow2(ports) ? ports - 1 : -1;
    a.rail_bits = a.N > 1 ? ilog2(a.N - 1) + 1 : 0;
    hipLaunchKernelGGL(port_tiles_kernel, dim3(1), dim3(1024), 0, st, a);
    if (int rc = launch_status()) return rc;
    hipLaunchKernelGGL(port_tile_kernel<false>, dim3(kPortBlocks), dim3(64 * kPortWaves), 0, st, a);
    if (int rc = launch_status()) return rc;
    hipLaunchKernelGGL(port_scan_kernel, dim3((unsigned)n_inst), dim3(64), 0, st, a);
    if (int rc = launch_status()) return rc;
    hipLaunchKernelGGL(port_tile_kernel<true>, dim3(kPortBlocks), dim3(64 * kPortWaves), 0, st, a);
    return launch_status();
}
