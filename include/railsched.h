/*
 * railsched - batched LPT rail spraying of MoE all-to-all traffic on one AMD MI355X (gfx950).
 *
 * C ABI of the hot path of RailS (arXiv 2510.19262): router logits -> top-k routing ->
 * GPU-to-GPU byte matrix D^(1) -> fixed-size chunks -> per-node descending sort ->
 * greedy least-loaded-rail assignment -> per-NIC send/receive loads, completion time,
 * lower bound.  The rails are simulated arithmetically; nothing is transmitted.
 *
 * Notation (Section 4.1, System Model): M domains (nodes); N GPUs = NICs = rails per domain;
 * G = M*N GPUs; GPU id g = d*N + n, 0-based; C = chunk bytes; R2 = rate of one rail.
 * "batch" is the number of independent traffic matrices (e.g. MoE layers) processed in one call;
 * an *instance* is one (matrix b, source node k) pair, numbered b*M + k.  Instances are scheduled
 * independently: each node decides from local information only (Sections 1 and 3.2).
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name starts with h_.  The caller owns every
 *     buffer (inputs, outputs, workspace); the library allocates nothing, keeps no state between
 *     calls (LoadState is reset for every all-to-all round, Section 5.2) and never frees anything.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All work is enqueued
 *     asynchronously on it; no call but railsched_check_capacity synchronises the host with the device.
 *   - Every function returns 0 (RAILSCHED_OK) or a negative railsched_status.  Arguments are
 *     validated on the host before anything is launched; on an error nothing has been enqueued.
 *   - All outputs are integers and are defined bit-exactly.
 *   - Capacity.  Every call that reads or writes the per-chunk arrays (chunk_w, chunk_flow, perm, rail, port) takes
 *     `capacity`, the number of records those arrays hold.  The chunk count chunk_off[batch*M] exists on the device
 *     only; when it exceeds `capacity` the call touches none of the per-chunk arrays and fills its remaining outputs
 *     with -1 instead (S for stage 4, R and stats for stage 5, all three for railsched_schedule), so a caller that
 *     never synchronises still finds the overflow in whatever it reads back; chunk_off is complete either way.
 *     railsched_check_capacity reports the same condition to the host as RAILSCHED_ERR_CAPACITY.
 *   - Limits: 1 <= N <= 64, 1 <= M, G <= 16384, N*G <= 16384 for chunk_sort, 1 <= k <= E <= 1024,
 *     1 <= C < 2^32, every instance holds fewer than 2^32 chunks and fewer than 2^56 bytes.
 */
#ifndef RAILSCHED_H
#define RAILSCHED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum railsched_status {
    RAILSCHED_OK = 0,
    RAILSCHED_ERR_INVALID_ARG = -1, /* a size or count is out of its documented range           */
    RAILSCHED_ERR_NULL_PTR    = -2, /* a required pointer is NULL                               */
    RAILSCHED_ERR_UNSUPPORTED = -3, /* valid in the paper's model but beyond this library's limits */
    RAILSCHED_ERR_CAPACITY    = -4, /* railsched_check_capacity: more chunks than the arrays hold */
    RAILSCHED_ERR_WORKSPACE   = -5, /* workspace missing or smaller than *_workspace_bytes()     */
    RAILSCHED_ERR_HIP         = -6, /* the HIP runtime refused a launch                          */
    RAILSCHED_ERR_SCRATCH     = -7  /* railsched_schedule_static: needs more than the static buffer */
} railsched_status;

/* Topology and chunking of the Rail fabric (Section 4.1; chunk size: Section 5.1, "Flow Splitting
 * and Atomicity").  Plain data, passed by HOST pointer. */
typedef struct railsched_topo {
    int32_t nodes;              /* M                                                             */
    int32_t rails;              /* N                                                             */
    int64_t chunk_bytes;        /* C                                                             */
    int64_t rail_bw_Bps;        /* R2 in bytes/s; only used by callers to turn bytes into time   */
    int32_t include_intra_node; /* 0: traffic inside a node is not inter-domain and is skipped   */
    int32_t reserved;           /* must be 0                                                     */
} railsched_topo_t;

const char *railsched_version(void);
const char *railsched_strerror(int status);

/* Waits until `stream` has drained, reads the chunk count chunk_off[batch*M] back and compares it with `capacity`
 * (Section 5.1: the number of atomic flows depends on the traffic, so record arrays sized ahead of time can turn
 * out too small).  The only call of the library that synchronises the host with the device.
 *   chunk_off [batch*M + 1] int64, as written by stage 3        (in)
 *   h_total   HOST pointer, receives the chunk count            (out, nullable)
 * Returns RAILSCHED_OK, RAILSCHED_ERR_CAPACITY (count > capacity; *h_total is still set), NULL_PTR, INVALID_ARG, HIP. */
int railsched_check_capacity(const int64_t *chunk_off, int32_t batch, const railsched_topo_t *h_topo, int64_t capacity,
                             int64_t *h_total, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 1 - gating decision (Algorithm 1 step 1; Top-K expert selection of Section 6.3).
 * For every token row the indices of the k largest logits, largest first; equal logits (IEEE
 * comparison, so -0 == +0) are ordered by ascending expert index.  Logits must be finite.
 *   logits   [rows][E] fp32, row-major            (in)
 *   topk_idx [rows][k] int32                      (out)
 * rows may be 0.  Errors: NULL_PTR, INVALID_ARG (rows < 0, E < 1, k < 1, k > E), UNSUPPORTED (E > 1024).
 * ------------------------------------------------------------------------------------------- */
int railsched_route_topk(const float *logits, int64_t rows, int32_t E, int32_t k,
                         int32_t *topk_idx, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 2 - GPU-to-GPU traffic matrix D^(1) (Section 4.1; Algorithm 1 step 2, selection of input
 * slices by gate and expert assignment).  Row r of matrix b belongs to source GPU
 * s = r / tokens_per_gpu; its slot j goes to GPU expert_gpu[topk_idx[r][j]][t mod R] with
 * t = r mod tokens_per_gpu (R replicas of every expert; R = 1 puts an expert on a single GPU);
 * every (token, slot) adds payload_bytes to D1[b][s][d].  A token whose slots hit the same GPU
 * counts once per slot.
 *   topk_idx   [batch*G*tokens_per_gpu][k] int32, values in [0,E)  (in; out-of-range values are ignored)
 *   expert_gpu [E][R] int32, values in [0,G)                        (in; same rule)
 *   D1         [batch][G][G] int64                                  (out, fully overwritten)
 *   ws         railsched_traffic_matrix_workspace_bytes(...) bytes of device memory, 4-byte aligned
 *              (scratch: destination counts of the slices a (matrix, source GPU) pair is cut into; summed in a
 *              fixed order by a second kernel, so no atomics leave the workgroups; contents undefined afterwards)
 * Errors: NULL_PTR, INVALID_ARG, UNSUPPORTED (G > 16384), WORKSPACE.
 * ------------------------------------------------------------------------------------------- */
size_t railsched_traffic_matrix_workspace_bytes(int32_t batch, int64_t tokens_per_gpu, int32_t k,
                                                const railsched_topo_t *h_topo);
int railsched_traffic_matrix(const int32_t *topk_idx, int32_t batch, int64_t tokens_per_gpu, int32_t k,
                             const int32_t *expert_gpu, int32_t E, int32_t R, int64_t payload_bytes,
                             const railsched_topo_t *h_topo, int64_t *D1, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stages 1 and 2 in one call (Algorithm 1 steps 1-2: gate, then selection of input slices by gate
 * and expert assignment).  Same inputs, same rules and bit-identical outputs as
 * railsched_route_topk over all batch*G*tokens_per_gpu rows followed by railsched_traffic_matrix;
 * for E <= 8 both are produced in a single pass over the logits and the indices are never read back; so is D1 for
 * 32 < E <= 256 with k <= 8 when the indices are not wanted (topk_idx == NULL; 16-byte aligned logits, E a multiple
 * of 4, G <= 4096); everything else runs the two stages.
 *   logits     [batch*G*tokens_per_gpu][E] fp32                     (in)
 *   expert_gpu [E][R] int32, values in [0,G)                        (in; out-of-range values are ignored)
 *   topk_idx   [batch*G*tokens_per_gpu][k] int32                    (out; may be NULL for the single-pass shapes:
 *                                                                    the picks are then counted but not stored)
 *   D1         [batch][G][G] int64                                  (out, fully overwritten)
 *   ws         railsched_route_traffic_workspace_bytes(...) bytes of device memory, 4-byte aligned
 *              (scratch: per-slice destination counts; contents undefined afterwards)
 * Errors: NULL_PTR (also topk_idx == NULL for a shape that runs the two stages), INVALID_ARG, UNSUPPORTED (E > 1024, G > 16384),
 * WORKSPACE (ws missing, misaligned or smaller than the query's answer).
 * ------------------------------------------------------------------------------------------- */
size_t railsched_route_traffic_workspace_bytes(int32_t batch, int64_t tokens_per_gpu, int32_t E, int32_t k,
                                               const railsched_topo_t *h_topo);
int railsched_route_traffic(const float *logits, int32_t batch, int64_t tokens_per_gpu, int32_t E, int32_t k,
                            const int32_t *expert_gpu, int32_t R, int64_t payload_bytes,
                            const railsched_topo_t *h_topo, int32_t *topk_idx, int64_t *D1, void *ws, size_t ws_bytes,
                            void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 3 - flow splitting and LPT sorting (Section 5.1 "Flow Splitting and Atomicity";
 * Algorithm 2 steps 1-2).  For instance (b,k) the flows of node k's N GPUs are taken in canonical
 * order (local GPU n ascending, destination GPU ascending; destinations inside node k skipped
 * unless include_intra_node); a flow of B bytes yields floor(B/C) chunks of C bytes and one of
 * B mod C bytes if that is non-zero.  The instance's chunks are then ordered by descending weight,
 * ties by source GPU, destination GPU and position in the flow (a stable sort of the canonical list).
 *   D1         [batch][G][G] int64, entries >= 0                     (in)
 *   chunk_off  [batch*M + 1] int64: exclusive scan of instance sizes (out)
 *   chunk_w    [capacity] uint32: chunk weight in bytes              (out, nullable)
 *   chunk_flow [capacity] uint32: n*G + destination GPU              (out)
 *   perm       [capacity] uint32: canonical position inside the instance of the chunk now at this
 *              sorted position                                      (out, nullable)
 * With chunk_w == NULL only chunk_off is produced (a count query: railsched_check_capacity then
 * returns the total to size the record arrays with).  If the total chunk count exceeds `capacity`
 * the record arrays are left untouched and chunk_off is still complete.
 * Workspace: railsched_chunk_sort_workspace_bytes(batch, topo) bytes, 256-byte aligned.
 * Errors: NULL_PTR, INVALID_ARG, UNSUPPORTED (N*G > 16384, C >= 2^32), WORKSPACE.
 * ------------------------------------------------------------------------------------------- */
size_t railsched_chunk_sort_workspace_bytes(int32_t batch, const railsched_topo_t *h_topo);
int railsched_chunk_sort(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo,
                         int64_t *chunk_off, uint32_t *chunk_w, uint32_t *chunk_flow, uint32_t *perm,
                         int64_t capacity, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 4 - LPT iterative allocation (Algorithm 2, initialisation and step 3).  Per instance:
 * LoadState[0..N) = 0; for every chunk in stored order j* = the lowest-numbered rail of minimum
 * LoadState; rail[i] = j*; LoadState[j*] += w_i.  The final LoadState is the send load S[b][k][.]
 * (Section 4.1, load matrix S).  Weights need not come from stage 3: any sequence is scheduled in
 * the order given (the guarantees of Theorem 4 need it non-increasing).
 *   chunk_off [batch*M + 1] int64   (in)
 *   chunk_w   [capacity] uint32     (in; the first chunk_off[batch*M] are read)
 *   rail      [capacity] uint8, values in [0,N)            (out; the first chunk_off[batch*M] are written)
 *   S         [batch][M][N] int64                          (out; every entry -1 if chunk_off[batch*M] > capacity,
 *                                                           and then chunk_w is not read and rail not written)
 *   ws        optional (NULL, 0 = none): railsched_lpt_spray_workspace_bytes(batch, topo) bytes, 256-byte aligned.
 *             Instances are independent (Sections 1 and 3.2), so the order they are worked on is free: with a
 *             workspace, batches of thousands of instances are taken longest chain first from a queue (the few far
 *             longer than the rest on a wavefront of their own), which evens out the load of the SIMDs; the outputs
 *             do not depend on it.  It pays for railsched_lpt_spray_chunkwise; railsched_lpt_spray, whose chains
 *             are what the closed forms leave over, accepts it and leaves it unused.
 * Errors: NULL_PTR, INVALID_ARG, UNSUPPORTED (N > 64), WORKSPACE (ws given but misaligned or too small).
 * ------------------------------------------------------------------------------------------- */
size_t railsched_lpt_spray_workspace_bytes(int32_t batch, const railsched_topo_t *h_topo);
int railsched_lpt_spray(const int64_t *chunk_off, const uint32_t *chunk_w, int32_t batch,
                        const railsched_topo_t *h_topo, int64_t capacity, uint8_t *rail, int64_t *S, void *ws,
                        size_t ws_bytes, void *stream);

/* Same function, same arguments, same outputs bit for bit (Algorithm 2 step 3), but every single chunk
 * goes through the cross-lane argmin; railsched_lpt_spray above additionally assigns whole periods of
 * equal-weight chunks in closed form when the rail loads are within one weight of each other (the
 * bound L_max <= L_opt + w_max of the Theorem 4 proof is what makes that state the common one).
 * Kept as the plain reference kernel for measurements and cross-checks. */
int railsched_lpt_spray_chunkwise(const int64_t *chunk_off, const uint32_t *chunk_w, int32_t batch,
                                  const railsched_topo_t *h_topo, int64_t capacity, uint8_t *rail, int64_t *S, void *ws,
                                  size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stage 5 - load evaluation (Section 4.1 load matrices S and R; Theorem 2; Theorem 3).
 * Rail n of a source node ends on NIC n of the destination node, so a chunk whose destination GPU
 * lies in node f and that was put on rail n adds its weight to R[b][f][n].
 *   R     [batch][M][N] int64                                   (out)
 *   stats [batch][8] int64                                      (out)
 *     [0] makespan = max over all entries of S[b] and R[b]  (Theorem 2: T = makespan / R2)
 *     [1] max send load   [2] max receive load
 *     [3] lower bound max( max_k ceil(sum_n S[b][k][n] / N), max_f ceil(sum_n R[b][f][n] / N), w_max )
 *         (uniform split of Theorem 3; one chunk is indivisible, Theorem 4 proof)
 *     [4] total bytes scheduled  [5] w_max  [6] chunk count
 *     [7] max over nodes k of (max_n S[b][k][n] - min_n S[b][k][n])
 * S is read as produced by stage 4.  No global atomics are used (the bins of a workgroup are
 * LDS-private integer atomics): every workgroup writes its partial receive loads to the workspace
 * and a second kernel adds them in a fixed order.
 * chunk_w, chunk_flow, rail hold `capacity` records; if chunk_off[batch*M] > capacity none of them is
 * read and every entry of R and stats is -1.
 * Workspace: railsched_eval_workspace_bytes(batch, topo) bytes, 256-byte aligned.
 * Errors: NULL_PTR, INVALID_ARG, UNSUPPORTED, WORKSPACE.
 * ------------------------------------------------------------------------------------------- */
size_t railsched_eval_workspace_bytes(int32_t batch, const railsched_topo_t *h_topo);
int railsched_eval(const int64_t *chunk_off, const uint32_t *chunk_w, const uint32_t *chunk_flow,
                   const uint8_t *rail, const int64_t *S, int32_t batch, const railsched_topo_t *h_topo,
                   int64_t capacity, int64_t *R, int64_t *stats, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Stages 3-5 in one call (Algorithm 2 steps 1-3 and 6; Section 4.1 S and R; Theorems 2-3): the outputs of
 * railsched_chunk_sort, railsched_lpt_spray and railsched_eval run one after the other on the same
 * arguments, bit for bit, with less work: stage 3 knows that every instance starts with a run of full chunks,
 * whose allocation from empty rails is round robin, so their rails are written with the records, stage 4 only
 * runs behind them and stage 5 takes their receive loads in closed form.  Batches of at most 1024 instances
 * with N*G <= 2048 flows and capacity <= 32768 chunks per instance are served by one workgroup per instance
 * (two launches after the counts instead of eight).
 *   D1 [batch][G][G] int64 (in);  chunk_off [batch*M+1];  chunk_w, chunk_flow, perm (perm may be NULL),
 *   rail: `capacity` records each;  S, R [batch][M][N] int64;  stats [batch][8] int64   (out)
 *   ws: railsched_schedule_workspace_bytes(batch, topo) bytes, 256-byte aligned.
 * If chunk_off[batch*M] > capacity the record arrays are left alone and every entry of S, R and stats is -1.
 * Errors: NULL_PTR, INVALID_ARG, UNSUPPORTED (as the three stages), WORKSPACE.
 * ------------------------------------------------------------------------------------------- */
size_t railsched_schedule_workspace_bytes(int32_t batch, const railsched_topo_t *h_topo);
int railsched_schedule(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo, int64_t *chunk_off,
                       uint32_t *chunk_w, uint32_t *chunk_flow, uint32_t *perm, int64_t capacity, uint8_t *rail,
                       int64_t *S, int64_t *R, int64_t *stats, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * railsched_schedule for callers that cannot allocate device memory or carry a workspace around: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments without the
 * workspace, same outputs bit for bit; the workspace is an array of RAILSCHED_STATIC_SCRATCH_BYTES bytes inside
 * the library's device image (every GPU the library runs on holds its own copy until the process ends).  The
 * call allocates and frees nothing; the first call on a device asks the runtime for the array's address there.
 * Batches whose railsched_schedule_workspace_bytes(batch, topo) exceeds RAILSCHED_STATIC_SCRATCH_BYTES are
 * refused with RAILSCHED_ERR_SCRATCH before anything is enqueued (4 MiB covers e.g. 32 matrices of 8 nodes x
 * 8 rails, or 1024 matrices of 4 x 4).
 * All calls on one GPU share that GPU's array: calls that can overlap there (different streams, or several
 * host threads) race on it and must be ordered by the caller; on one stream they are ordered already.
 * Errors: as railsched_schedule without WORKSPACE, plus SCRATCH, and HIP when the device has no such array.
 * ------------------------------------------------------------------------------------------- */
#define RAILSCHED_STATIC_SCRATCH_BYTES (4u << 20)
int railsched_schedule_static(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo, int64_t *chunk_off,
                              uint32_t *chunk_w, uint32_t *chunk_flow, uint32_t *perm, int64_t capacity, uint8_t *rail,
                              int64_t *S, int64_t *R, int64_t *stats, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Second all-to-all of an MoE layer (Algorithm 1 step 4: expert outputs return to the token owners):
 * its traffic is the first one's reversed, D1T[b][d][s] = D1[b][s][d]; stages 3-5 then run on D1T.
 *   D1, D1T [batch][G][G] int64, distinct buffers.
 * Errors: NULL_PTR, INVALID_ARG (also D1 == D1T), UNSUPPORTED.
 * ------------------------------------------------------------------------------------------- */
int railsched_transpose_matrix(const int64_t *D1, int32_t batch, const railsched_topo_t *h_topo, int64_t *D1T,
                               void *stream);

/* ---------------------------------------------------------------------------------------------
 * The path-selection schemes RailS is compared with (Sections 1, 2.2 and 6.1), reduced to arithmetic
 * on the chunk records of stage 3: same inputs and outputs as stage 4, another rule for the rail.
 *   RAILSCHED_POLICY_NIC_DIRECT   a GPU's traffic leaves through its own NIC: rail = flow id div G
 *   RAILSCHED_POLICY_FLOW_HASH    static per-flow hashing (ECMP-like): hash(instance*N*G + flow id) mod N
 *   RAILSCHED_POLICY_RANDOM_SPRAY per chunk: hash(index of the chunk in the record arrays) mod N
 *   RAILSCHED_POLICY_ROUND_ROBIN  chunk i of the instance, in stored order, takes rail i mod N
 * hash(x) = splitmix64 finaliser of (seed + 0x9E3779B97F4A7C15 * (x + 1)), 64-bit wrapping.
 *   rail [capacity] uint8 (out), S [batch][M][N] int64 send loads (out); feed both to railsched_eval.
 * If chunk_off[batch*M] > capacity the per-chunk arrays are left alone and every entry of S is -1.
 * Errors: NULL_PTR, INVALID_ARG (unknown policy), UNSUPPORTED.
 * ------------------------------------------------------------------------------------------- */
enum { RAILSCHED_POLICY_NIC_DIRECT = 0, RAILSCHED_POLICY_FLOW_HASH = 1, RAILSCHED_POLICY_RANDOM_SPRAY = 2,
       RAILSCHED_POLICY_ROUND_ROBIN = 3 };
int railsched_assign_policy(int32_t policy, uint64_t seed, const int64_t *chunk_off, const uint32_t *chunk_w,
                            const uint32_t *chunk_flow, int32_t batch, const railsched_topo_t *h_topo,
                            int64_t capacity, uint8_t *rail, int64_t *S, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Spraying execution, port choice (Algorithm 2 step 4: round-robin port choice inside the chosen NIC):
 * each rail of a node hands its chunks to its `ports` queue pairs in turn; the chunk that is the c-th
 * one (c = 0, 1, ...) put on its rail inside its instance, in stored order, takes port c mod ports.
 *   rail [chunks] uint8 (in), port [chunks] uint8 (out), 1 <= ports <= 256.
 * `capacity` is the number of records rail and port hold and sizes the workspace:
 * railsched_port_round_robin_workspace_bytes(batch, topo, capacity) bytes, 256-byte aligned.
 * If chunk_off[batch*M] exceeds capacity, rail is not read and port not written.
 * Errors: NULL_PTR, INVALID_ARG, UNSUPPORTED (ports > 256), WORKSPACE.
 * ------------------------------------------------------------------------------------------- */
size_t railsched_port_round_robin_workspace_bytes(int32_t batch, const railsched_topo_t *h_topo, int64_t capacity);
int railsched_port_round_robin(const int64_t *chunk_off, const uint8_t *rail, int32_t batch,
                               const railsched_topo_t *h_topo, int32_t ports, int64_t capacity, uint8_t *port,
                               void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RAILSCHED_H */
