/*
 * CPU oracle for the rail-spraying hot path of RailS (arXiv 2510.19262).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * single-purpose restatement of what the pipeline computes, written from the
 * paper, and it shares no code, header, table or helper with the GPU library.
 * Only the test-suite, the smoke check and the CPU-baseline leg of the
 * benchmark may call it.
 *
 * Notation (Section 4.1, System Model): M domains (nodes), N GPUs = NICs =
 * rails per domain, G = M*N GPUs, GPU id g = d*N + n (0-based here), C = chunk
 * bytes, D1 = GPU-to-GPU byte matrix D^(1), D2 = domain-to-domain matrix D^(2).
 *
 * LPT is a heuristic, so the oracle is the algorithm taken step by step
 * (Algorithm 2, initialisation, steps 1-3 and 6) with these tie-breaks, which
 * make exactly one result correct:
 *   - top-k: experts ordered by (logit descending, index ascending) under IEEE
 *     comparison (so -0 and +0 tie); the first k indices in that order;
 *   - sort: weight descending, ties by source GPU index (Algorithm 2, step 2),
 *     then destination GPU, then position inside the flow, i.e. a stable sort
 *     of the canonical enumeration;
 *   - argmin: the lowest rail index among the minima.
 *
 * Pins (tests/test_oracle_*.py): numpy's stable argsort for top-k and sort,
 * byte conservation and closed-form one-hot routing for the matrix, brute-force
 * optimal assignment and Graham's bound (Theorem 4 proof), the textbook tight
 * LPT family, equal weights => round robin, the greedy max-min <= w_max
 * invariant, a second min-heap LPT, rail conservation, and the exact uniform
 * receive loads of Theorem 3 on all-equal inputs.
 * "Normalized MSE" (Section 6.1, metrics) has no printed formula: parity unpinned
 * for that one derived quantity; the raw MSE of Algorithm 2 step 6 is pinned.
 *
 * All byte quantities are int64; weights of single chunks are uint32.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_MAX_E 4096
#define ORACLE_MAX_N 64

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* threads the parallel loops use from now on (n < 1: as many as the runtime offers); returns the count in force */
int oracle_set_threads(int n)
{
#ifdef _OPENMP
    omp_set_num_threads(n < 1 ? omp_get_num_procs() : n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}

/* ------------------------------------------------------------------------
 * Step 1 (Algorithm 1 step 1, "Gate"; Top-K of Section 6.3): for every token
 * row the k experts with the largest router logit, best first.  The j-th
 * output is the largest remaining logit; among equal logits the lowest index.
 * ---------------------------------------------------------------------- */
int oracle_route_topk(const float *logits, int64_t rows, int E, int k, int32_t *topk_idx)
{
    if (E < 1 || E > ORACLE_MAX_E || k < 1 || k > E || rows < 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *x = logits + r * (int64_t)E;
        unsigned char taken[ORACLE_MAX_E];
        memset(taken, 0, (size_t)E);
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || x[e] > x[best]) best = e;
            }
            taken[best] = 1;
            topk_idx[r * (int64_t)k + j] = best;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Step 2 (Algorithm 1 step 2, where every expert's input slices are picked by
 * the gate and the expert placement; D^(1) of Section 4.1): every (token,
 * slot) sends payload bytes from the token's GPU to the GPU hosting the chosen
 * expert.  Row r of a layer lives on GPU s = r / tokens_per_gpu; replica rho =
 * (r mod tokens_per_gpu) mod R of the expert receives it.
 * D1 is [batch][G][G] and is overwritten.
 * ---------------------------------------------------------------------- */
int oracle_traffic_matrix(const int32_t *topk_idx, int batch, int64_t tokens_per_gpu, int k,
                          const int32_t *expert_gpu, int E, int R, int64_t payload_bytes,
                          int M, int N, int64_t *D1)
{
    const int64_t G = (int64_t)M * N;
    memset(D1, 0, sizeof(int64_t) * (size_t)batch * G * G);
    int err = 0;
#pragma omp parallel for schedule(static) reduction(min : err)
    for (int64_t bs = 0; bs < (int64_t)batch * G; ++bs) {      /* bs = b*G + s */
        for (int64_t t = 0; t < tokens_per_gpu; ++t) {
            const int64_t r = bs * tokens_per_gpu + t;
            const int rho = (int)(t % R);
            for (int j = 0; j < k; ++j) {
                const int32_t e = topk_idx[r * k + j];
                if (e < 0 || e >= E) { err = -2; continue; }
                const int32_t d = expert_gpu[(int64_t)e * R + rho];
                if (d < 0 || d >= G) { err = -3; continue; }
                D1[bs * G + d] += payload_bytes;
            }
        }
    }
    return err;
}

/* D^(2)_{d,f} = sum_n sum_m D^(1)_{(d,n),(f,m)}  (Section 4.1, eq. 1). One matrix. */
void oracle_domain_matrix(const int64_t *D1, int M, int N, int64_t *D2)
{
    const int64_t G = (int64_t)M * N;
    for (int d = 0; d < M; ++d)
        for (int f = 0; f < M; ++f) {
            int64_t acc = 0;
            for (int n = 0; n < N; ++n)
                for (int m = 0; m < N; ++m)
                    acc += D1[((int64_t)d * N + n) * G + ((int64_t)f * N + m)];
            D2[(int64_t)d * M + f] = acc;
        }
}

/* ------------------------------------------------------------------------
 * Step 3a (flow splitting, Section 5.1 "Flow Splitting and Atomicity"): a
 * GPU-to-GPU flow of B bytes becomes floor(B/C) chunks of C bytes plus one of
 * B mod C bytes when that is non-zero.  Source node k emits the flows of its N
 * GPUs in canonical order: local GPU n ascending, destination GPU ascending,
 * position in the flow ascending.  Traffic that stays inside node k is not
 * inter-domain and is skipped unless include_intra is set.
 * flow id = n*G + dst.  With w == NULL only counts.  Returns the chunk count.
 * ---------------------------------------------------------------------- */
int64_t oracle_chunk_split(const int64_t *D1mat, int M, int N, int64_t C, int include_intra,
                           int node, uint32_t *w, uint32_t *flow)
{
    const int64_t G = (int64_t)M * N;
    int64_t cnt = 0;
    for (int n = 0; n < N; ++n) {
        const int64_t src = (int64_t)node * N + n;
        for (int64_t dst = 0; dst < G; ++dst) {
            if (!include_intra && dst / N == node) continue;
            const int64_t B = D1mat[src * G + dst];
            const int64_t full = B / C;
            const int64_t rem = B % C;
            for (int64_t q = 0; q < full; ++q) {
                if (w) { w[cnt] = (uint32_t)C; flow[cnt] = (uint32_t)(n * G + dst); }
                ++cnt;
            }
            if (rem > 0) {
                if (w) { w[cnt] = (uint32_t)rem; flow[cnt] = (uint32_t)(n * G + dst); }
                ++cnt;
            }
        }
    }
    return cnt;
}

/* ------------------------------------------------------------------------
 * Step 3b (Algorithm 2 step 2): sort by descending weight; equal weights keep
 * their canonical order.  perm[sorted position] = canonical position.
 * The C library sort is the primitive; the comparator is a total order, so the
 * result is the stable sort.
 * ---------------------------------------------------------------------- */
typedef struct { uint32_t w, flow, pos; } rec_t;

static int rec_cmp(const void *a, const void *b)
{
    const rec_t *x = (const rec_t *)a, *y = (const rec_t *)b;
    if (x->w != y->w) return x->w > y->w ? -1 : 1;
    if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
    return 0;
}

int oracle_sort_desc(int64_t n, uint32_t *w, uint32_t *flow, uint32_t *perm)
{
    if (n <= 0) return 0;
    rec_t *r = (rec_t *)malloc(sizeof(rec_t) * (size_t)n);
    if (!r) return -1;
    for (int64_t i = 0; i < n; ++i) { r[i].w = w[i]; r[i].flow = flow[i]; r[i].pos = (uint32_t)i; }
    qsort(r, (size_t)n, sizeof(rec_t), rec_cmp);
    for (int64_t i = 0; i < n; ++i) {
        w[i] = r[i].w; flow[i] = r[i].flow;
        if (perm) perm[i] = r[i].pos;
    }
    free(r);
    return 0;
}

/* ------------------------------------------------------------------------
 * Step 4 (Algorithm 2, initialisation and step 3): LoadState[0..N) = 0; for
 * each flow in the given order j* = argmin_j LoadState[j] (lowest j among
 * minima); record j*; LoadState[j*] += w.  L returns the final LoadState.
 * ---------------------------------------------------------------------- */
void oracle_lpt(int64_t n, const uint32_t *w, int N, uint8_t *rail, int64_t *L)
{
    for (int j = 0; j < N; ++j) L[j] = 0;
    for (int64_t i = 0; i < n; ++i) {
        int js = 0;
        for (int j = 1; j < N; ++j)
            if (L[j] < L[js]) js = j;
        rail[i] = (uint8_t)js;
        L[js] += (int64_t)w[i];
    }
}

/* The same rule through a binary min-heap ordered by (load, rail): an
 * independent second implementation used to cross-check the scan above. */
typedef struct { int64_t load; int rail; } hnode_t;

static int h_less(const hnode_t *a, const hnode_t *b)
{
    return a->load < b->load || (a->load == b->load && a->rail < b->rail);
}

static void h_sift_down(hnode_t *h, int n, int i)
{
    for (;;) {
        int l = 2 * i + 1, r = l + 1, m = i;
        if (l < n && h_less(&h[l], &h[m])) m = l;
        if (r < n && h_less(&h[r], &h[m])) m = r;
        if (m == i) return;
        hnode_t t = h[i]; h[i] = h[m]; h[m] = t;
        i = m;
    }
}

void oracle_lpt_heap(int64_t n, const uint32_t *w, int N, uint8_t *rail, int64_t *L)
{
    hnode_t h[ORACLE_MAX_N];
    for (int j = 0; j < N; ++j) { h[j].load = 0; h[j].rail = j; }  /* already a heap */
    for (int64_t i = 0; i < n; ++i) {
        rail[i] = (uint8_t)h[0].rail;
        h[0].load += (int64_t)w[i];
        h_sift_down(h, N, 0);
    }
    for (int j = 0; j < N; ++j) L[h[j].rail] = h[j].load;
}

/* Exact optimal makespan of n weights on N rails by exhaustive enumeration
 * (N^n assignments; tiny inputs only).  The reference for Graham's ratio. */
static void opt_rec(int i, int n, const uint32_t *w, int N, int64_t *L, int64_t *best)
{
    if (i == n) {
        int64_t mx = 0;
        for (int j = 0; j < N; ++j) if (L[j] > mx) mx = L[j];
        if (mx < *best) *best = mx;
        return;
    }
    for (int j = 0; j < N; ++j) {
        L[j] += w[i];
        opt_rec(i + 1, n, w, N, L, best);
        L[j] -= w[i];
    }
}

int64_t oracle_opt_makespan(int n, const uint32_t *w, int N)
{
    int64_t L[ORACLE_MAX_N];
    int64_t best = INT64_MAX;
    for (int j = 0; j < N; ++j) L[j] = 0;
    opt_rec(0, n, w, N, L, &best);
    return best;
}

/* ------------------------------------------------------------------------
 * Step 5 (Section 4.1 load matrices S and R; Theorem 2; Theorem 3): for ONE
 * matrix.  Rail n of source node k ends on NIC n of the destination node
 * (Theorem 3 proof), so a chunk with destination GPU dst on rail n adds to
 * R[dst / N][n].  chunk_off is this matrix's M+1 offsets into the record
 * arrays.  Ssum is recomputed from the records (send side), R from the same
 * records (receive side).
 *   stats[0] makespan = max over all S and R entries   (Theorem 2, times R2)
 *   stats[1] max send load, stats[2] max receive load
 *   stats[3] lower bound max( max_k ceil(out_k/N), max_f ceil(in_f/N), w_max )
 *            (uniform split of Theorem 3; a chunk is indivisible)
 *   stats[4] total bytes, stats[5] w_max, stats[6] chunk count
 *   stats[7] max over nodes of (max_n S[k][n] - min_n S[k][n])
 * ---------------------------------------------------------------------- */
/* stats[0..8) of one matrix from its load matrices, its largest chunk weight and its chunk count */
static void stats_from_loads(const int64_t *S, const int64_t *R, int64_t wmax, int64_t chunks, int M, int N, int64_t *stats)
{
    int64_t max_s = 0, max_r = 0, lb = wmax, total = 0, spread = 0;
    for (int k = 0; k < M; ++k) {
        int64_t out = 0, in = 0, smin = INT64_MAX, smax = 0;
        for (int n = 0; n < N; ++n) {
            const int64_t s = S[(int64_t)k * N + n], r = R[(int64_t)k * N + n];
            out += s; in += r;
            if (s > max_s) max_s = s;
            if (r > max_r) max_r = r;
            if (s < smin) smin = s;
            if (s > smax) smax = s;
        }
        total += out;
        if ((out + N - 1) / N > lb) lb = (out + N - 1) / N;
        if ((in + N - 1) / N > lb) lb = (in + N - 1) / N;
        if (smax - smin > spread) spread = smax - smin;
    }
    stats[0] = max_s > max_r ? max_s : max_r;
    stats[1] = max_s;
    stats[2] = max_r;
    stats[3] = lb;
    stats[4] = total;
    stats[5] = wmax;
    stats[6] = chunks;
    stats[7] = spread;
}

void oracle_eval(const int64_t *chunk_off, const uint32_t *w, const uint32_t *flow,
                 const uint8_t *rail, int M, int N, int64_t *Ssum, int64_t *R, int64_t *stats)
{
    const int64_t G = (int64_t)M * N;
    for (int64_t i = 0; i < (int64_t)M * N; ++i) { Ssum[i] = 0; R[i] = 0; }
    int64_t wmax = 0;
    for (int k = 0; k < M; ++k) {
        for (int64_t i = chunk_off[k]; i < chunk_off[k + 1]; ++i) {
            const int64_t dst = (int64_t)flow[i] % G;
            const int f = (int)(dst / N);
            Ssum[(int64_t)k * N + rail[i]] += (int64_t)w[i];
            R[(int64_t)f * N + rail[i]] += (int64_t)w[i];
            if ((int64_t)w[i] > wmax) wmax = (int64_t)w[i];
        }
    }
    stats_from_loads(Ssum, R, wmax, chunk_off[M] - chunk_off[0], M, N, stats);
}

/* ------------------------------------------------------------------------
 * One whole traffic matrix taken one source node at a time, for matrices whose chunk records do not fit
 * in host memory together: node k's flows are split (Section 5.1), sorted and allocated (Algorithm 2
 * steps 2-3) by the functions above, its final LoadState is S[k][.], and the weight of each of its chunks
 * is added to R[f][rail] of the chunk's destination node f (Section 4.1; rail n ends on NIC n of the
 * destination, Theorem 3 proof); the records are then dropped.  Node k's receive contributions are kept
 * apart until all nodes are done and added in node order.  Same S, R, stats and chunk_off[0..M] as
 * chunk_sort_batch -> lpt_batch -> eval on the matrix.  Returns 0, or -1 when memory runs out.
 * ---------------------------------------------------------------------- */
int oracle_schedule_matrix_by_node(const int64_t *D1mat, int M, int N, int64_t C, int include_intra,
                                   int64_t *chunk_off, int64_t *S, int64_t *R, int64_t *stats)
{
    const int64_t G = (int64_t)M * N;
    int64_t *Rk = (int64_t *)calloc((size_t)M * (size_t)G, sizeof(int64_t));     /* [k][f][n] */
    int64_t *cnt = (int64_t *)calloc((size_t)M, sizeof(int64_t));
    int64_t *wmax_k = (int64_t *)calloc((size_t)M, sizeof(int64_t));
    if (!Rk || !cnt || !wmax_k) { free(Rk); free(cnt); free(wmax_k); return -1; }
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(min : err)
    for (int k = 0; k < M; ++k) {
        const int64_t n = oracle_chunk_split(D1mat, M, N, C, include_intra, k, NULL, NULL);
        cnt[k] = n;
        uint32_t *w = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(n > 0 ? n : 1));
        uint32_t *flow = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(n > 0 ? n : 1));
        uint8_t *rail = (uint8_t *)malloc((size_t)(n > 0 ? n : 1));
        if (!w || !flow || !rail || oracle_sort_desc(oracle_chunk_split(D1mat, M, N, C, include_intra, k, w, flow), w, flow, NULL)) {
            err = -1;
        } else {
            oracle_lpt(n, w, N, rail, S + (int64_t)k * N);
            for (int64_t i = 0; i < n; ++i) {
                const int f = (int)(((int64_t)flow[i] % G) / N);
                Rk[(int64_t)k * G + (int64_t)f * N + rail[i]] += (int64_t)w[i];
                if ((int64_t)w[i] > wmax_k[k]) wmax_k[k] = (int64_t)w[i];
            }
        }
        free(w); free(flow); free(rail);
    }
    int64_t wmax = 0;
    chunk_off[0] = 0;
    for (int64_t i = 0; i < G; ++i) R[i] = 0;
    for (int k = 0; k < M; ++k) {
        chunk_off[k + 1] = chunk_off[k] + cnt[k];
        if (wmax_k[k] > wmax) wmax = wmax_k[k];
        for (int64_t i = 0; i < G; ++i) R[i] += Rk[(int64_t)k * G + i];
    }
    if (!err) stats_from_loads(S, R, wmax, chunk_off[M], M, N, stats);
    free(Rk); free(cnt); free(wmax_k);
    return err;
}

/* ------------------------------------------------------------------------
 * Batched drivers: the same steps over every (matrix, source node) instance.
 * Instances are independent (each node schedules from local information only,
 * Section 1 / Section 3.2), hence the plain parallel-for.
 * ---------------------------------------------------------------------- */

/* chunk_off[batch*M + 1]: exclusive scan of the per-instance chunk counts. */
void oracle_chunk_count_batch(const int64_t *D1, int batch, int M, int N, int64_t C,
                              int include_intra, int64_t *chunk_off)
{
    const int64_t G = (int64_t)M * N;
    const int64_t inst = (int64_t)batch * M;
    int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)(inst > 0 ? inst : 1));
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < inst; ++i)
        cnt[i] = oracle_chunk_split(D1 + (i / M) * G * G, M, N, C, include_intra, (int)(i % M), NULL, NULL);
    chunk_off[0] = 0;
    for (int64_t i = 0; i < inst; ++i) chunk_off[i + 1] = chunk_off[i] + cnt[i];
    free(cnt);
}

/* Split, then sort every instance in place inside the batch-wide record arrays. */
int oracle_chunk_sort_batch(const int64_t *D1, int batch, int M, int N, int64_t C, int include_intra,
                            const int64_t *chunk_off, uint32_t *w, uint32_t *flow, uint32_t *perm)
{
    const int64_t G = (int64_t)M * N;
    const int64_t inst = (int64_t)batch * M;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(min : err)
    for (int64_t i = 0; i < inst; ++i) {
        const int64_t o = chunk_off[i];
        const int64_t n = oracle_chunk_split(D1 + (i / M) * G * G, M, N, C, include_intra, (int)(i % M),
                                             w + o, flow + o);
        if (n != chunk_off[i + 1] - o) { err = -1; continue; }
        if (oracle_sort_desc(n, w + o, flow + o, perm ? perm + o : NULL)) err = -2;
    }
    return err;
}

void oracle_lpt_batch(const int64_t *chunk_off, const uint32_t *w, int batch, int M, int N,
                      uint8_t *rail, int64_t *S)
{
    const int64_t inst = (int64_t)batch * M;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < inst; ++i) {
        const int64_t o = chunk_off[i];
        oracle_lpt(chunk_off[i + 1] - o, w + o, N, rail + o, S + i * N);
    }
}

void oracle_eval_batch(const int64_t *chunk_off, const uint32_t *w, const uint32_t *flow,
                       const uint8_t *rail, int batch, int M, int N,
                       int64_t *Ssum, int64_t *R, int64_t *stats)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < batch; ++b)
        oracle_eval(chunk_off + (int64_t)b * M, w, flow, rail, M, N,
                    Ssum + (int64_t)b * M * N, R + (int64_t)b * M * N, stats + (int64_t)b * 8);
}

/* ------------------------------------------------------------------------
 * Second all-to-all (Algorithm 1 step 4, expert outputs back to the token owners): every byte
 * sent from GPU s to GPU d in the first all-to-all returns from d to s, so the traffic matrix of
 * the second one is the transpose, matrix by matrix: D1T[b][d][s] = D1[b][s][d].
 * ---------------------------------------------------------------------- */
void oracle_transpose_batch(const int64_t *D1, int batch, int64_t G, int64_t *D1T)
{
    for (int b = 0; b < batch; ++b)
        for (int64_t s = 0; s < G; ++s)
            for (int64_t d = 0; d < G; ++d)
                D1T[((int64_t)b * G + d) * G + s] = D1[((int64_t)b * G + s) * G + d];
}

/* ------------------------------------------------------------------------
 * Arithmetic stand-ins for the path-selection schemes RailS is compared with (Sections 1, 2.2 and
 * 6.1): the same chunk records, a different rule for the rail of each chunk.
 *   0 NIC-direct : no spraying, a GPU's traffic leaves through its own NIC: rail = source local GPU
 *                  (flow id div G).  Rails used directly, with no multipath transport.
 *   1 flow hash  : static per-flow hashing as in ECMP: every chunk of a GPU-to-GPU flow takes the rail
 *                  hash(instance, flow id) mod N.
 *   2 random spray: every chunk independently, hash(position of the chunk in the record arrays) mod N.
 *   3 round robin : chunk i of the instance (in stored order) takes rail i mod N, blind to sizes.
 * hash(x) = splitmix64 finaliser of (seed + 0x9E3779B97F4A7C15 * (x + 1)).
 * S receives the per-rail send loads of the instance.
 * ---------------------------------------------------------------------- */
static uint64_t o_mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

static uint64_t o_hash(uint64_t seed, uint64_t x)
{
    return o_mix64(seed + 0x9E3779B97F4A7C15ull * (x + 1));
}

int oracle_assign_policy(int policy, uint64_t seed, const int64_t *chunk_off, const uint32_t *w,
                         const uint32_t *flow, int batch, int M, int N, uint8_t *rail, int64_t *S)
{
    const int64_t G = (int64_t)M * N, NF = (int64_t)N * G;
    const int64_t inst_n = (int64_t)batch * M;
    if (policy < 0 || policy > 3) return -1;
    for (int64_t inst = 0; inst < inst_n; ++inst) {
        int64_t *L = S + inst * N;
        for (int n = 0; n < N; ++n) L[n] = 0;
        for (int64_t i = chunk_off[inst]; i < chunk_off[inst + 1]; ++i) {
            int r;
            switch (policy) {
                case 0: r = (int)(flow[i] / G); break;
                case 1: r = (int)(o_hash(seed, (uint64_t)inst * (uint64_t)NF + flow[i]) % (uint64_t)N); break;
                case 2: r = (int)(o_hash(seed, (uint64_t)i) % (uint64_t)N); break;
                default: r = (int)((i - chunk_off[inst]) % N); break;
            }
            rail[i] = (uint8_t)r;
            L[r] += (int64_t)w[i];
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Spraying execution, port choice (Algorithm 2 step 4: round-robin port choice inside the chosen NIC):
 * every rail of a node hands its chunks to its P ports (queue pairs) in turn, so the chunk that is
 * the c-th one put on its rail within its instance (c = 0, 1, ...) takes port c mod P.
 * ---------------------------------------------------------------------- */
void oracle_port_round_robin(const int64_t *chunk_off, const uint8_t *rail, int batch, int M, int N, int P,
                             uint8_t *port)
{
    const int64_t inst_n = (int64_t)batch * M;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t inst = 0; inst < inst_n; ++inst) {
        int64_t seen[ORACLE_MAX_N];
        for (int n = 0; n < N; ++n) seen[n] = 0;
        for (int64_t i = chunk_off[inst]; i < chunk_off[inst + 1]; ++i) {
            port[i] = (uint8_t)(seen[rail[i]] % P);
            seen[rail[i]] += 1;
        }
    }
}
