"""Seeded sweep over random small shapes: every entry point against the CPU oracle, bit for bit.
The fixed cases of test_gpu_parity.py pin known corners; this sweep looks for the unknown ones."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_19262_amd as rs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _random_stack(rng, B, G, C):
    kind = int(rng.integers(0, 4))
    if kind == 0:       # mixed full chunks and tails
        m = rng.integers(0, int(rng.integers(2, 9)) * C, size=(B, G, G))
    elif kind == 1:     # tails only
        m = rng.integers(0, max(C, 2), size=(B, G, G))
    elif kind == 2:     # whole chunks only, few distinct sizes
        m = rng.integers(0, 4, size=(B, G, G)) * C
    else:               # payload-like: multiples of a granule
        gran = max(C // int(rng.integers(2, 33)), 1)
        m = rng.integers(0, 200, size=(B, G, G)) * gran
    m = m.astype(np.int64)
    m[rng.random((B, G, G)) < rng.random() * 0.9] = 0
    return m


@pytest.mark.parametrize("seed", range(40))
def test_random_shape_stages_3_to_5_both_ways(seed):
    rng = np.random.default_rng(1000 + seed)
    N = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 24, 32, 48, 64]))
    M = int(rng.integers(1, max(2, min(9, 1024 // (N * N) + 2))))
    B = int(rng.integers(1, 6)) if seed % 5 else int(rng.integers(100, 400))
    if B > 50:
        N, M = min(N, 4), min(M, 4)
    C = int(rng.choice([1, 7, 64, 1000, 4096, 65536, 262144]))
    intra = int(rng.integers(0, 2))
    perm = bool(rng.integers(0, 2))
    G = M * N
    D1n = _random_stack(rng, B, G, C)
    topo = rs.Topo(M, N, C, include_intra_node=intra)
    D1 = torch.from_numpy(D1n).to(DEV)

    off_c, w_c, flow_c, perm_c = oracle.chunk_sort_batch(D1n, M, N, C, intra)
    rail_c, S_c = oracle.lpt_batch(off_c, w_c, B, M, N)
    _, R_c, stats_c = oracle.eval_batch(off_c, w_c, flow_c, rail_c, B, M, N)
    n = int(off_c[-1])

    def check(off, w, flow, pm, rail, S, R, stats, what):
        assert np.array_equal(off.cpu().numpy(), off_c), what
        assert np.array_equal(_u32(w)[:n], w_c) and np.array_equal(_u32(flow)[:n], flow_c), what
        if pm is not None:
            assert np.array_equal(_u32(pm)[:n], perm_c), what
        assert np.array_equal(rail.cpu().numpy()[:n], rail_c), what
        assert np.array_equal(S.cpu().numpy(), S_c) and np.array_equal(R.cpu().numpy(), R_c), what
        assert np.array_equal(stats.cpu().numpy(), stats_c), what

    off, w, flow, pm = rs.chunk_sort(D1, topo, want_perm=perm)
    rail, S = rs.lpt_spray(off, w, B, topo)
    R, stats = rs.eval(off, w, flow, rail, S, B, topo)
    check(off, w, flow, pm, rail, S, R, stats, f"three calls M={M} N={N} B={B} C={C}")
    slack = int(rng.integers(0, 3)) * int(rng.integers(0, 100000))
    out = rs.schedule(D1, topo, n + slack, want_perm=perm)
    check(*out, f"one call M={M} N={N} B={B} C={C} capacity +{slack}")
    rail2, S2 = rs.lpt_spray(off, w, B, topo, chunkwise=True)
    assert torch.equal(rail2[:n], rail[:n]) and torch.equal(S2, S)


@pytest.mark.parametrize("seed", range(30))
def test_random_shape_routing_both_ways(seed):
    rng = np.random.default_rng(2000 + seed)
    E = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 8, 8, 12, 16, 32, 40, 64, 100, 128, 256]))
    k = int(rng.integers(1, min(E, 9) + 1))
    N = int(rng.choice([1, 2, 4, 8]))
    M = int(rng.integers(1, 5))
    G = M * N
    R = int(rng.choice([1, 2, 3, 4, 8]))
    tok = int(rng.choice([0, 1, 7, 255, 256, 511, 513, 1000, 4099]))
    batch = int(rng.integers(1, 4))
    rows = batch * G * tok
    lattice = bool(rng.integers(0, 2))
    x = ((rng.integers(-8, 9, size=(rows, E)) * 0.125) if lattice else rng.standard_normal((rows, E))).astype(np.float32)
    eg = rng.integers(0, G, size=(E, R)).astype(np.int32)
    topo = rs.Topo(M, N, 4096)
    want_idx = oracle.route_topk(x, k) if rows else np.empty((0, k), np.int32)
    want_D1 = oracle.traffic_matrix(want_idx, batch, tok, eg, 1536, M, N)
    xd, egd = torch.from_numpy(x).to(DEV).view(rows, E), torch.from_numpy(eg).to(DEV)
    idx = rs.route_topk(xd, k)
    assert np.array_equal(idx.cpu().numpy(), want_idx), f"route_topk E={E} k={k}"
    D1 = rs.traffic_matrix(idx, batch, tok, egd, 1536, topo)
    assert np.array_equal(D1.cpu().numpy(), want_D1), f"traffic_matrix E={E} k={k} R={R} tok={tok}"
    idx2, D12 = rs.route_traffic(xd, k, batch, tok, egd, 1536, topo)
    assert np.array_equal(idx2.cpu().numpy(), want_idx) and np.array_equal(D12.cpu().numpy(), want_D1), f"route_traffic E={E} k={k}"
