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

__device__ __forceinline__ int pol_last_le(const int64_t *v, int n, int64_t x)
{
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (v[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void fill_zero_kernel(int64_t *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// Streaming over all chunk positions, four per thread at multiples of four.  Send loads go to LDS bins
// for the first kPolSlots instances a tile touches (a tile rarely touches more) and from there, or
// directly for the rest, to S with integer atomics (S is zeroed first; integer sums are order-free).
__global__ __launch_bounds__(kPolThreads) void policy_kernel(PolArgs a)
{
    __shared__ int64_t s_off[kPolStage + 1];
    __shared__ unsigned long long bins[kPolSlots][kMaxRails];
    const int64_t total = a.chunk_off[a.n_inst];
    for (int64_t t0 = (int64_t)blockIdx.x * kPolTile; t0 < total; t0 += (int64_t)gridDim.x * kPolTile) {
        const int64_t t1 = t0 + kPolTile < total ? t0 + kPolTile : total;
        const int inst_lo = pol_last_le(a.chunk_off, a.n_inst, t0);
        const int inst_hi = pol_last_le(a.chunk_off, a.n_inst, t1 - 1);
        const int cnt = inst_hi - inst_lo + 1;
        const bool staged = cnt <= kPolStage;
        __syncthreads();                                   // previous tile is done with the LDS
        if (staged)
            for (int i = threadIdx.x; i <= cnt; i += kPolThreads) s_off[i] = a.chunk_off[inst_lo + i];
        for (int i = threadIdx.x; i < kPolSlots * kMaxRails; i += kPolThreads) (&bins[0][0])[i] = 0ull;
        __syncthreads();
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
            int li = staged ? pol_last_le(s_off, cnt, p) : pol_last_le(a.chunk_off, a.n_inst, p) - inst_lo;
            uint32_t packed = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (p + e >= total) break;
                int64_t nxt = staged ? s_off[li + 1] : a.chunk_off[inst_lo + li + 1];
                while (p + e >= nxt) { ++li; nxt = staged ? s_off[li + 1] : a.chunk_off[inst_lo + li + 1]; }
                const int64_t b = staged ? s_off[li] : a.chunk_off[inst_lo + li];
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
        __syncthreads();
        for (int i = threadIdx.x; i < kPolSlots * a.N; i += kPolThreads) {
            const int li = i / a.N, r = i % a.N;
            const unsigned long long v = bins[li][r];
            if (v && li < cnt) atomicAdd(reinterpret_cast<unsigned long long *>(a.S + (int64_t)(inst_lo + li) * a.N + r), v);
        }
    }
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
                                       uint8_t *rail, int64_t *S, void *stream)
{
    using namespace rs;
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0 || policy < 0 || policy > 3) return RAILSCHED_ERR_INVALID_ARG;
    const int64_t n_inst = (int64_t)batch * h_topo->nodes;
    if (n_inst > 0x7FFFFFFFll / 64) return RAILSCHED_ERR_UNSUPPORTED;
    if (n_inst == 0) return RAILSCHED_OK;
    if (!chunk_off || !S) return RAILSCHED_ERR_NULL_PTR;
    hipStream_t st = static_cast<hipStream_t>(stream);
    PolArgs a;
    a.chunk_off = chunk_off; a.chunk_w = chunk_w; a.chunk_flow = chunk_flow; a.rail = rail; a.S = S; a.seed = seed;
    a.n_inst = (int32_t)n_inst; a.N = h_topo->rails; a.G = h_topo->nodes * h_topo->rails; a.NF = a.N * a.G; a.policy = policy;
    a.nmask = is_pow2(a.N) ? a.N - 1 : -1;
    a.gshift = is_pow2(a.G) ? ilog2(a.G) : -1;
    a.wide_ok = (reinterpret_cast<uintptr_t>(chunk_w) % 16 == 0 && reinterpret_cast<uintptr_t>(chunk_flow) % 16 == 0 &&
                 reinterpret_cast<uintptr_t>(rail) % 4 == 0) ? 1 : 0;
    const int64_t n = n_inst * a.N;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n + 255) / 256 > 1024 ? 1024 : (n + 255) / 256)), dim3(256), 0, st, S, n);
    if (int rc = launch_status()) return rc;
    hipLaunchKernelGGL(policy_kernel, dim3(kPolBlocks), dim3(kPolThreads), 0, st, a);
    return launch_status();
}
