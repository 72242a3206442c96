"""Pins for the CPU oracle: every function is checked against something other than
itself - a library routine with the same definition, a closed form, an invariant,
brute force on tiny inputs, or a hand-worked fixture under tests/golden/.
No GPU is needed and nothing here touches the HIP library.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as W


def _read_golden(path):
    out = {}
    flows = []
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            vals = [int(v) for v in vals]
            if key == "flow":
                flows.append(vals)
            else:
                out[key] = vals
    out["flow"] = flows
    return out


# ------------------------------------------------------------------ top-k
def _topk_by_stable_sort(logits, k):
    # full stable sort of the indices by descending logit (numpy's stable argsort on the negation)
    return np.argsort(-logits.astype(np.float64), axis=1, kind="stable")[:, :k].astype(np.int32)


@pytest.mark.parametrize("E,k", [(8, 2), (8, 8), (8, 1), (5, 3), (256, 8), (64, 6), (1, 1), (300, 7)])
def test_topk_equals_full_stable_sort(E, k):
    rng = np.random.default_rng(E * 131 + k)
    # few distinct values => many exact ties
    logits = rng.integers(-3, 4, size=(257, E)).astype(np.float32) * np.float32(0.5)
    assert np.array_equal(oracle.route_topk(logits, k), _topk_by_stable_sort(logits, k))
    logits = rng.standard_normal((129, E)).astype(np.float32)
    assert np.array_equal(oracle.route_topk(logits, k), _topk_by_stable_sort(logits, k))


def test_topk_special_cases():
    E = 8
    rng = np.random.default_rng(1)
    x = rng.standard_normal((64, E)).astype(np.float32)
    full = oracle.route_topk(x, E)
    assert np.array_equal(np.sort(full, axis=1), np.tile(np.arange(E), (64, 1)))      # k=E: a permutation
    assert np.array_equal(oracle.route_topk(x, 1)[:, 0], np.argmax(x, axis=1))        # k=1: first argmax
    allsame = np.full((3, E), 1.25, dtype=np.float32)
    assert np.array_equal(oracle.route_topk(allsame, 3), np.tile(np.arange(3), (3, 1)))
    dup = np.array([[0, 5, 1, 5, 5, -1, 2, 0]], dtype=np.float32)
    assert oracle.route_topk(dup, 4).tolist() == [[1, 3, 4, 6]]
    pmz = np.array([[-1, -0.0, 0.0, -2, 0.0, -0.0, -3, -4]], dtype=np.float32)       # -0 == +0 tie
    assert oracle.route_topk(pmz, 4).tolist() == [[1, 2, 4, 5]]


def test_topk_on_workload_logits():
    cfg = W.get_config("c1")
    x = W.gen_logits(cfg, 0, rows=4096).numpy()
    assert np.array_equal(oracle.route_topk(x, cfg.k), _topk_by_stable_sort(x, cfg.k))


# ------------------------------------------------------------------ traffic matrix
def _routing(cfg, rows_scale=1):
    x = W.gen_logits(cfg, 0).numpy()
    idx = oracle.route_topk(x, cfg.k)
    eg = W.expert_gpu_table(cfg)
    D1 = oracle.traffic_matrix(idx, 1, cfg.tokens_per_gpu, eg, cfg.payload_bytes, cfg.M, cfg.N)
    return x, idx, eg, D1


def test_traffic_matrix_conservation_and_rows():
    cfg = W.get_config("c1")
    _, idx, eg, D1 = _routing(cfg)
    per_gpu = cfg.tokens_per_gpu * cfg.k * cfg.payload_bytes
    assert D1.shape == (1, cfg.G, cfg.G)
    assert D1.sum() == cfg.G * per_gpu                                   # byte conservation
    assert np.all(D1[0].sum(axis=1) == per_gpu)                          # every source GPU sends the same
    # independent recount with numpy: destination of every (token, slot)
    t_local = np.arange(cfg.rows_per_layer) % cfg.tokens_per_gpu
    src = np.arange(cfg.rows_per_layer) // cfg.tokens_per_gpu
    dst = eg[idx, (t_local % eg.shape[1])[:, None]]
    ref = np.zeros((cfg.G, cfg.G), dtype=np.int64)
    np.add.at(ref, (np.repeat(src, cfg.k), dst.reshape(-1)), cfg.payload_bytes)
    assert np.array_equal(D1[0], ref)
    assert not np.array_equal(D1[0], D1[0].T)                            # a transposed result would differ


def test_traffic_matrix_one_hot():
    # one expert far ahead: all first-choice bytes land on that expert's R replica GPUs,
    # split by t_local mod R (ceil/floor closed form)
    M, N, E, R, tok, payload = 2, 3, 3, 2, 7, 100
    G = M * N
    eg = np.array([[0, 3], [1, 4], [2, 5]], dtype=np.int32)
    logits = np.zeros((G * tok, E), dtype=np.float32)
    logits[:, 1] = 100.0
    idx = oracle.route_topk(logits, 1)
    D1 = oracle.traffic_matrix(idx, 1, tok, eg, payload, M, N)[0]
    expect = np.zeros((G, G), dtype=np.int64)
    expect[:, 1] = payload * ((tok + 1) // 2)       # t_local even -> replica 0
    expect[:, 4] = payload * (tok // 2)             # t_local odd  -> replica 1
    assert np.array_equal(D1, expect)


def test_traffic_matrix_batch_layers_independent():
    M, N, E, k, tok = 2, 2, 4, 2, 5
    G = M * N
    rng = np.random.default_rng(3)
    eg = rng.integers(0, G, size=(E, 2)).astype(np.int32)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(3 * G * tok)]).astype(np.int32)
    D = oracle.traffic_matrix(idx, 3, tok, eg, 8, M, N)
    for b in range(3):
        Db = oracle.traffic_matrix(idx[b * G * tok:(b + 1) * G * tok], 1, tok, eg, 8, M, N)
        assert np.array_equal(D[b], Db[0])


def test_domain_matrix_is_block_sum():
    M, N = 3, 4
    rng = np.random.default_rng(5)
    D1 = rng.integers(0, 1000, size=(M * N, M * N)).astype(np.int64)
    D2 = oracle.domain_matrix(D1, M, N)
    assert np.array_equal(D2, D1.reshape(M, N, M, N).sum(axis=(1, 3)))


# ------------------------------------------------------------------ chunk split and sort
def _rand_matrix(rng, G, C, p_zero=0.3):
    m = rng.integers(0, 6 * C, size=(G, G)).astype(np.int64)
    m[rng.random((G, G)) < p_zero] = 0
    m[rng.random((G, G)) < 0.2] //= C
    m[rng.random((G, G)) < 0.2] = 3 * C              # exact multiples: no tail chunk
    return m


@pytest.mark.parametrize("include_intra", [0, 1])
def test_chunk_split_per_flow(include_intra):
    M, N, C = 3, 2, 64
    G = M * N
    rng = np.random.default_rng(7)
    D1 = _rand_matrix(rng, G, C)
    for node in range(M):
        w, flow = oracle.chunk_split(D1, M, N, C, node, include_intra)
        assert np.all(w <= C) and np.all(w > 0)
        assert np.all(np.diff(flow.astype(np.int64)) >= 0)                # canonical order: flow ids ascend
        for n in range(N):
            for dst in range(G):
                sel = w[flow == n * G + dst]
                B = int(D1[node * N + n, dst])
                if dst // N == node and not include_intra:
                    assert sel.size == 0
                    continue
                assert int(sel.sum()) == B                                 # bytes of the flow are conserved
                assert sel.size == -(-B // C)                              # ceil(B/C) chunks
                assert np.count_nonzero(sel < C) <= 1                      # at most one tail
                if sel.size:
                    assert np.all(sel[:-1] == C)                           # tail is last


def test_chunk_offsets_are_exclusive_scan():
    M, N, C = 3, 2, 64
    rng = np.random.default_rng(8)
    D1 = np.stack([_rand_matrix(rng, M * N, C) for _ in range(4)])
    off = oracle.chunk_count_batch(D1, M, N, C)
    counts = [oracle.chunk_split(D1[b], M, N, C, k)[0].size for b in range(4) for k in range(M)]
    assert off[0] == 0 and np.array_equal(np.diff(off), counts)


def test_sort_equals_numpy_stable_sort():
    rng = np.random.default_rng(9)
    for n in (0, 1, 2, 17, 1000):
        w = rng.integers(1, 9, size=n).astype(np.uint32)
        flow = rng.integers(0, 50, size=n).astype(np.uint32)
        sw, sf, perm = oracle.sort_desc(w, flow)
        ref = np.argsort(-w.astype(np.int64), kind="stable")
        assert np.array_equal(perm, ref)
        assert np.array_equal(sw, w[ref]) and np.array_equal(sf, flow[ref])
        assert np.all(np.diff(sw.astype(np.int64)) <= 0)
        assert np.array_equal(np.sort(perm), np.arange(n))


def test_batched_sort_matches_per_instance():
    M, N, C = 4, 2, 32
    rng = np.random.default_rng(10)
    D1 = np.stack([_rand_matrix(rng, M * N, C) for _ in range(3)])
    off, w, flow, perm = oracle.chunk_sort_batch(D1, M, N, C)
    for b in range(3):
        for k in range(M):
            cw, cf = oracle.chunk_split(D1[b], M, N, C, k)
            ref = np.argsort(-cw.astype(np.int64), kind="stable")
            o, e = off[b * M + k], off[b * M + k + 1]
            assert np.array_equal(w[o:e], cw[ref]) and np.array_equal(flow[o:e], cf[ref])
            assert np.array_equal(perm[o:e], ref)


# ------------------------------------------------------------------ LPT
def _greedy_python(w, N):
    L = [0] * N
    rails = []
    for x in w:
        j = min(range(N), key=lambda q: (L[q], q))
        rails.append(j)
        L[j] += int(x)
    return rails, L


def test_lpt_graham_tight_fixture(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "lpt_graham_tight_n3.txt"))
    N = g["N"][0]
    rail, L = oracle.lpt(np.array(g["weights"], dtype=np.uint32), N)
    assert rail.tolist() == g["rails"] and L.tolist() == g["loads"]
    assert L.max() == g["lpt_makespan"][0]
    assert oracle.opt_makespan(np.array(g["weights"], dtype=np.uint32), N) == g["opt_makespan"][0]


@pytest.mark.parametrize("N", [2, 3, 4])
def test_lpt_tight_family(N):
    # 2N-1,2N-1,...,N+1,N+1,N,N,N : LPT = 4N-1, OPT = 3N  (ratio exactly 4/3 - 1/(3N))
    w = [v for x in range(2 * N - 1, N, -1) for v in (x, x)] + [N, N, N]
    rail, L = oracle.lpt(np.array(w, dtype=np.uint32), N)
    assert L.max() == 4 * N - 1
    assert oracle.opt_makespan(np.array(w, dtype=np.uint32), N) == 3 * N


def test_lpt_vs_brute_force_optimum():
    rng = np.random.default_rng(11)
    for trial in range(60):
        N = int(rng.integers(2, 5))
        n = int(rng.integers(1, 10 if N < 4 else 9))
        w = np.sort(rng.integers(1, 30, size=n).astype(np.uint32))[::-1].copy()
        rail, L = oracle.lpt(w, N)
        opt = oracle.opt_makespan(w, N)
        # independent optimum by itertools enumeration
        best = min(max(sum(int(w[i]) for i in range(n) if a[i] == j) for j in range(N))
                   for a in itertools.product(range(N), repeat=n)) if N ** n <= 70000 else opt
        assert opt == best
        assert opt <= L.max()
        assert 3 * N * int(L.max()) <= (4 * N - 1) * opt                 # Graham's ratio, in integers
        assert int(L.max()) <= -(-int(w.sum()) // N) + int(w.max())      # L_max <= L_opt + w_max


def test_lpt_equal_weights_is_round_robin():
    for N in (1, 2, 4, 8, 5):
        for F in (0, 1, N - 1, N, 3 * N + 2, 100):
            if F < 0:
                continue
            w = np.full(F, 4096, dtype=np.uint32)
            rail, L = oracle.lpt(w, N)
            assert np.array_equal(rail, np.arange(F) % N)
            assert L.sum() == 4096 * F


def test_lpt_small_cases():
    rail, L = oracle.lpt(np.array([9, 7, 3], dtype=np.uint32), 1)
    assert rail.tolist() == [0, 0, 0] and L.tolist() == [19]
    rail, L = oracle.lpt(np.array([9, 7, 3], dtype=np.uint32), 5)         # F <= N: chunk i on rail i
    assert rail.tolist() == [0, 1, 2] and L.tolist() == [9, 7, 3, 0, 0]
    rail, L = oracle.lpt(np.array([], dtype=np.uint32), 4)
    assert rail.size == 0 and L.tolist() == [0, 0, 0, 0]


def test_lpt_invariants_and_second_implementation():
    rng = np.random.default_rng(12)
    for N in (2, 4, 8, 3, 64):
        for n in (1, 50, 3000):
            w = np.sort(rng.integers(1, 1 << 18, size=n).astype(np.uint32))[::-1].copy()
            w[rng.random(n) < 0.5] = w[0]                                 # long runs of equal weights
            w = np.sort(w)[::-1].copy()
            rail, L = oracle.lpt(w, N)
            rail2, L2 = oracle.lpt(w, N, heap=True)                             # independent min-heap version
            assert np.array_equal(rail, rail2) and np.array_equal(L, L2)
            if n <= 50:
                r3, L3 = _greedy_python(w, N)                              # and a plain Python restatement
                assert rail.tolist() == r3 and L.tolist() == L3
            assert np.array_equal(L, np.bincount(rail, weights=w.astype(np.float64), minlength=N).astype(np.int64))
            wmax, tot = int(w.max()), int(w.sum())
            assert int(L.max() - L.min()) <= wmax                          # greedy keeps max-min <= w_max
            assert all(abs(Fraction(int(x)) - Fraction(tot, N)) <= wmax for x in L)
            assert oracle.load_mse(L) <= wmax * wmax                       # Theorem 4
            assert int(L.max()) <= -(-tot // N) + wmax


def test_lpt_max_minus_min_holds_at_every_step():
    rng = np.random.default_rng(13)
    w = np.sort(rng.integers(1, 1000, size=200).astype(np.uint32))[::-1].copy()
    N = 4
    rail, _ = oracle.lpt(w, N)
    L = np.zeros(N, dtype=np.int64)
    for i in range(w.size):
        assert rail[i] == int(np.argmin(L))                                # numpy argmin: first minimum
        L[rail[i]] += int(w[i])
        assert L.max() - L.min() <= int(w[0])


def test_mse_definition():
    assert oracle.load_mse([11, 8, 8]) == Fraction(2)                      # mean 9: (4+1+1)/3
    assert oracle.load_mse([5, 5, 5, 5]) == 0
    assert oracle.load_mse([12, 0, 0, 0], normalized=True) == 1
    assert oracle.load_mse([3, 3, 3, 3], normalized=True) == 0


# ------------------------------------------------------------------ eval
def _pipeline(D1, M, N, C, include_intra=0):
    D1 = np.asarray(D1, dtype=np.int64)
    if D1.ndim == 2:
        D1 = D1[None]
    B = D1.shape[0]
    off, w, flow, perm = oracle.chunk_sort_batch(D1, M, N, C, include_intra)
    rail, S = oracle.lpt_batch(off, w, B, M, N)
    Ssum, R, stats = oracle.eval_batch(off, w, flow, rail, B, M, N)
    return off, w, flow, perm, rail, S, Ssum, R, stats


def test_eval_single_flow_fixture(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "single_flow_receive.txt"))
    M, N, C = g["M"][0], g["N"][0], g["C"][0]
    G = M * N
    D1 = np.zeros((G, G), dtype=np.int64)
    for d, n, f, m, nbytes in g["flow"]:
        D1[d * N + n, f * N + m] = nbytes
    off, w, flow, perm, rail, S, Ssum, R, stats = _pipeline(D1, M, N, C)
    assert off.tolist() == [0, 6, 6, 6]
    assert w.tolist() == g["sorted_w"] and flow.tolist() == g["sorted_flow"]
    assert perm.tolist() == g["perm"] and rail.tolist() == g["rails"]
    assert S[0, 0].tolist() == g["S0"] and Ssum[0, 0].tolist() == g["S0"]
    assert R[0, 1].tolist() == g["R1"] and R[0, 2].tolist() == g["R2"] and R[0, 0].tolist() == [0, 0]
    assert stats[0, 0] == g["makespan"][0] and stats[0, 3] == g["lower_bound"][0]
    assert stats[0].tolist() == [25, 25, 20, 24, 47, 10, 6, 3]


def test_schedule_matrix_by_node_pins(golden_dir):
    # the node-at-a-time form used for matrices too large to hold: the hand-worked fixture, the closed form of the
    # all-equal matrix (Theorem 3) and, on random matrices with and without intra-node traffic, the batched steps
    g = _read_golden(os.path.join(golden_dir, "single_flow_receive.txt"))
    M, N, C = g["M"][0], g["N"][0], g["C"][0]
    D1 = np.zeros((M * N, M * N), dtype=np.int64)
    for d, n, f, m, nbytes in g["flow"]:
        D1[d * N + n, f * N + m] = nbytes
    off, S, R, stats = oracle.schedule_matrix_by_node(D1, M, N, C)
    assert off.tolist() == [0, 6, 6, 6] and S[0].tolist() == g["S0"] and R.tolist() == [[0, 0], g["R1"], g["R2"]]
    assert stats.tolist() == [25, 25, 20, 24, 47, 10, 6, 3]
    for (M, N, q) in [(4, 4, 3), (5, 3, 2)]:
        C = 4096
        off, S, R, stats = oracle.schedule_matrix_by_node(W.symmetric_matrix(M, N, q, C), M, N, C)
        expect = (M - 1) * N * q * C
        assert np.all(S == expect) and np.all(R == expect) and stats[0] == stats[3] == expect and stats[7] == 0
        assert off.tolist() == [k * (M - 1) * N * N * q for k in range(M + 1)]
    rng = np.random.default_rng(21)
    for (M, N, C, intra) in [(6, 4, 1000, 0), (3, 5, 64, 1), (9, 2, 4096, 0)]:
        D1 = rng.integers(0, 7 * C, size=(M * N, M * N)).astype(np.int64)
        D1[rng.random(D1.shape) < 0.3] = 0
        off, S, R, stats = oracle.schedule_matrix_by_node(D1, M, N, C, intra)
        b_off, b_w, b_flow, _ = oracle.chunk_sort_batch(D1[None], M, N, C, intra)
        b_rail, b_S = oracle.lpt_batch(b_off, b_w, 1, M, N)
        _, b_R, b_stats = oracle.eval_batch(b_off, b_w, b_flow, b_rail, 1, M, N)
        assert np.array_equal(off, b_off) and np.array_equal(S, b_S[0]) and np.array_equal(R, b_R[0]) and np.array_equal(stats, b_stats[0])


def test_eval_conservation_on_workload():
    cfg = W.get_config("c1")
    _, _, _, D1 = _routing(cfg)
    M, N, C = cfg.M, cfg.N, cfg.chunk_bytes
    off, w, flow, perm, rail, S, Ssum, R, stats = _pipeline(D1, M, N, C)
    assert np.array_equal(S, Ssum)                                         # LoadState == recomputed send loads
    D2 = oracle.domain_matrix(D1[0], M, N)
    offdiag = D2 - np.diag(np.diag(D2))
    assert np.array_equal(S[0].sum(axis=1), offdiag.sum(axis=1))           # sum_n S[k][n] = sum_{f!=k} D2[k][f]
    assert np.array_equal(R[0].sum(axis=1), offdiag.sum(axis=0))           # sum_n R[f][n] = sum_{k!=f} D2[k][f]
    assert np.array_equal(S[0].sum(axis=0), R[0].sum(axis=0))              # per-rail conservation
    st = stats[0]
    assert st[0] == max(S.max(), R.max()) and st[1] == S.max() and st[2] == R.max()
    assert st[4] == offdiag.sum() and st[5] == w.max() and st[6] == w.size
    lb = max(max(-(-int(x) // N) for x in offdiag.sum(axis=1)),
             max(-(-int(x) // N) for x in offdiag.sum(axis=0)), int(w.max()))
    assert st[3] == lb and st[0] >= st[3]
    assert st[7] == (S[0].max(axis=1) - S[0].min(axis=1)).max() <= w.max()
    # with intra-node traffic kept, the full D2 is scheduled
    off2, w2, *_rest = _pipeline(D1, M, N, C, include_intra=1)
    assert int(w2.astype(np.int64).sum()) == int(D1.sum())


def test_eval_uniform_send_gives_uniform_receive():
    # all-equal matrix, entries q*C: every (source GPU, destination node) block is N*q equal
    # chunks in a row, so LPT splits it evenly and R[f][n] = S[k][n] = (M-1)*N*q*C exactly
    for (M, N, q) in [(4, 4, 3), (3, 2, 1), (5, 8, 2)]:
        C = 4096
        D1 = W.symmetric_matrix(M, N, q, C)
        off, w, flow, perm, rail, S, Ssum, R, stats = _pipeline(D1, M, N, C)
        expect = (M - 1) * N * q * C
        assert np.all(S == expect) and np.all(R == expect)
        assert stats[0, 0] == stats[0, 3] == expect                         # makespan == lower bound
        assert stats[0, 7] == 0


def test_eval_receive_can_be_uneven_when_send_is_even():
    # discrete LPT balances a node's total send only; a single tiny example where R is not uniform
    M, N, C = 2, 2, 10
    D1 = np.zeros((4, 4), dtype=np.int64)
    D1[0, 2] = 10
    D1[1, 3] = 10
    *_x, S, Ssum, R, stats = _pipeline(D1, M, N, C)
    assert S[0, 0].tolist() == [10, 10] and R[0, 1].tolist() == [10, 10]
    D1[1, 3] = 0
    D1[0, 2] = 10
    *_x, S, Ssum, R, stats = _pipeline(D1, M, N, C)
    assert S[0, 0].tolist() == [10, 0] and R[0, 1].tolist() == [10, 0]


def test_flows_workload_shape():
    cfg = W.get_config("c3").scaled(M=4, batch=2)
    D1 = W.gen_flow_matrices(cfg)
    assert D1.shape == (2, 32, 32) and np.all(np.diagonal(D1, axis1=1, axis2=2) == 0)
    assert np.all(D1 % 4096 == 0)
    assert 0.55 < (D1 == 0).mean() < 0.85
    again = W.gen_flow_matrices(cfg, first=1, count=1)
    assert np.array_equal(again[0], D1[1])                                  # counter based: order independent


# ------------------------------------------------------------------ second all-to-all, comparison schemes
def test_transpose_is_numpy_transpose():
    rng = np.random.default_rng(21)
    D1 = rng.integers(0, 1 << 40, size=(3, 12, 12)).astype(np.int64)
    T = oracle.transpose_batch(D1)
    assert np.array_equal(T, np.transpose(D1, (0, 2, 1)))
    assert np.array_equal(oracle.transpose_batch(T), D1)
    assert not np.array_equal(T, D1)


def _records(seed=22, M=4, N=4, C=4096, B=2):
    rng = np.random.default_rng(seed)
    D1 = _rand_matrix(rng, M * N, C)[None].repeat(B, axis=0)
    D1[1] = _rand_matrix(rng, M * N, C)
    off, w, flow, perm = oracle.chunk_sort_batch(D1, M, N, C)
    return D1, off, w, flow, M, N, B


def test_policy_nic_direct_is_the_row_sum():
    # without spraying a GPU's inter-node bytes all leave on its own NIC: S[b][k][n] = row sum of GPU (k,n)
    D1, off, w, flow, M, N, B = _records()
    rail, S = oracle.assign_policy("nic_direct", 0, off, w, flow, B, M, N)
    G = M * N
    inter = D1.copy()
    for k in range(M):
        inter[:, k * N:(k + 1) * N, k * N:(k + 1) * N] = 0
    assert np.array_equal(S.reshape(B, G), inter.sum(axis=2))
    assert np.array_equal(rail, (flow // G).astype(np.uint8))


def test_policy_round_robin_closed_form():
    D1, off, w, flow, M, N, B = _records()
    rail, S = oracle.assign_policy("round_robin", 0, off, w, flow, B, M, N)
    for inst in range(B * M):
        o, e = off[inst], off[inst + 1]
        assert np.array_equal(rail[o:e], np.arange(e - o) % N)
        assert np.array_equal(S.reshape(-1, N)[inst], np.bincount(rail[o:e], weights=w[o:e].astype(np.float64), minlength=N).astype(np.int64))


def _hash_np(seed, x):
    with np.errstate(over="ignore"):
        return W.mix64_np(np.uint64(seed) + np.uint64(0x9E3779B97F4A7C15) * (x.astype(np.uint64) + np.uint64(1)))


def test_policy_hashes_match_a_numpy_restatement():
    D1, off, w, flow, M, N, B = _records()
    G, NF = M * N, N * M * N
    seed = 12345
    rail, S = oracle.assign_policy("flow_hash", seed, off, w, flow, B, M, N)
    inst = np.repeat(np.arange(B * M), np.diff(off))
    assert np.array_equal(rail, (_hash_np(seed, inst.astype(np.uint64) * np.uint64(NF) + flow) % np.uint64(N)).astype(np.uint8))
    for i in range(B * M):                                   # a flow never changes rail
        o, e = off[i], off[i + 1]
        for f in np.unique(flow[o:e]):
            assert np.unique(rail[o:e][flow[o:e] == f]).size == 1
    rail2, S2 = oracle.assign_policy("random_spray", seed, off, w, flow, B, M, N)
    assert np.array_equal(rail2, (_hash_np(seed, np.arange(w.size)) % np.uint64(N)).astype(np.uint8))
    counts = np.bincount(rail2, minlength=N)
    assert counts.min() > 0.8 * w.size / N and counts.max() < 1.2 * w.size / N      # roughly uniform
    for r, s_ in ((rail, S), (rail2, S2)):
        for i in range(B * M):
            o, e = off[i], off[i + 1]
            assert np.array_equal(s_.reshape(-1, N)[i], np.bincount(r[o:e], weights=w[o:e].astype(np.float64), minlength=N).astype(np.int64))
    assert not np.array_equal(oracle.assign_policy("random_spray", seed + 1, off, w, flow, B, M, N)[0], rail2)


def test_lpt_is_never_worse_than_the_lower_bound_and_beats_blind_schemes_on_skew():
    # one hot GPU per node: NIC-direct piles everything on one rail, LPT spreads it
    M, N, C = 4, 4, 4096
    G = M * N
    D1 = np.full((1, G, G), C, dtype=np.int64)
    for k in range(M):
        D1[0, k * N, :] = 40 * C + 123
    off, w, flow, perm = oracle.chunk_sort_batch(D1, M, N, C)
    rail_l, S_l = oracle.lpt_batch(off, w, 1, M, N)
    st_l = oracle.eval_batch(off, w, flow, rail_l, 1, M, N)[2][0]
    rail_d, S_d = oracle.assign_policy("nic_direct", 0, off, w, flow, 1, M, N)
    st_d = oracle.eval_batch(off, w, flow, rail_d, 1, M, N)[2][0]
    assert st_l[3] == st_d[3] and st_l[0] >= st_l[3]
    assert st_d[0] > 2 * st_l[0]


def test_port_round_robin():
    import pandas as pd
    D1, off, w, flow, M, N, B = _records(seed=31)
    rail, _ = oracle.lpt_batch(off, w, B, M, N)
    inst = np.repeat(np.arange(B * M), np.diff(off))
    for P in (1, 3, 4, 256):
        port = oracle.port_round_robin(off, rail, B, M, N, P)
        ref = pd.DataFrame({"i": inst, "r": rail}).groupby(["i", "r"]).cumcount().to_numpy() % P   # library cumulative count
        assert np.array_equal(port, ref.astype(np.uint8))
    assert not oracle.port_round_robin(off, rail, B, M, N, 1).any()
    # equal weights: rail = i mod N, so the port is (i div N) mod P
    off2 = np.array([0, 50], dtype=np.int64)
    rail2, _ = oracle.lpt(np.full(50, 7, dtype=np.uint32), 4)
    assert np.array_equal(oracle.port_round_robin(off2, rail2, 1, 1, 4, 3), (np.arange(50) // 4) % 3)


# ------------------------------------------------------------------ facts the GPU kernels' shortcuts rest on
@pytest.mark.parametrize("N", [2, 3, 4, 8, 13])
def test_lpt_run_of_equal_weights_visits_rails_in_load_order(N):
    """A run of one weight w entered with max - min load < w goes round after round through the rails in
    ascending (load, rail) order (the premise of Theorem 4's equal-granularity bound, used as a closed form
    by the kernels).  The entry loads are made by N descending chunks, which land on rails 0..N-1."""
    rng = np.random.default_rng(N)
    for trial in range(30):
        w = int(rng.integers(50, 1000))
        loads = np.sort(rng.integers(1000, 1000 + w, size=N))[::-1].astype(np.uint32)      # spread < w, descending
        L = int(rng.integers(1, 5 * N))
        weights = np.concatenate([loads, np.full(L, w, dtype=np.uint32)])
        rail, final = oracle.lpt(weights, N)
        assert list(rail[:N]) == list(range(N))
        order = sorted(range(N), key=lambda j: (int(loads[j]), j))
        assert list(rail[N:]) == [order[i % N] for i in range(L)]
        want = [int(loads[j]) + w * (L // N + (order.index(j) < L % N)) for j in range(N)]
        assert list(final) == want


@pytest.mark.parametrize("N", [1, 2, 3, 8, 40])
def test_round_robin_share_of_a_position_range(N):
    """Positions s..e-1 of a round-robin run put (e+N-1-n) div N - (s+N-1-n) div N chunks on rail n: the closed
    form the one-call scheduler uses for the receive loads of an instance's leading run."""
    rng = np.random.default_rng(100 + N)
    for trial in range(200):
        s = int(rng.integers(0, 500))
        e = s + int(rng.integers(0, 300))
        for n in range(N):
            brute = sum(1 for i in range(s, e) if i % N == n)
            assert (e + N - 1 - n) // N - (s + N - 1 - n) // N == brute


def test_leading_run_of_a_sorted_instance_is_round_robin_with_equal_loads():
    """Stage 3 puts all full chunks (weight C) first; from empty rails their first n_full - n_full mod N go
    i mod N and leave every rail with C * (n_full div N): what the one-call scheduler starts stage 4 from."""
    rng = np.random.default_rng(5)
    M, N, C = 3, 4, 1000
    G = M * N
    D1 = rng.integers(0, 7 * C, size=(G, G)).astype(np.int64)
    for k in range(M):
        w, flow = oracle.chunk_split(D1, M, N, C, k)
        sw, sf, _ = oracle.sort_desc(w, flow)
        n_full = int((sw == C).sum())
        assert np.all(sw[:n_full] == C) and np.all(sw[n_full:] < C)
        lead = n_full - n_full % N
        rail, _ = oracle.lpt(sw, N)
        assert np.array_equal(rail[:lead], np.arange(lead) % N)
        _, loads = oracle.lpt(sw[:lead], N)
        assert np.all(loads == C * (n_full // N))
