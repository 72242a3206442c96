"""The hand-worked fixtures under tests/golden/ and the closed-form uniform workload, through the C ABI end to end.

Expected values here come from the fixture files (worked by hand from the paper's definitions) and from the
closed form of the all-equal matrix (the discrete instance of Theorem 3), not from any implementation; the
oracle is compared as well, so a disagreement names the side that is wrong.
"""
import os

import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

rs = pytest.importorskip("paper_2510_19262_amd")
DEV = "cuda:0"


def _read_golden(path):
    out, flows = {}, []
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


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _paths(D1_np, topo):
    """Stages 3-5 three ways: the three calls, the three calls with the per-chunk LPT kernel, the one call.
    Yields (name, dict of numpy outputs)."""
    D1 = torch.from_numpy(np.ascontiguousarray(D1_np)).to(DEV)
    B = D1.shape[0]
    for name in ("three calls", "three calls, per-chunk kernel", "one call"):
        if name == "one call":
            total = rs.chunk_total(D1, topo)
            off, w, flow, perm, rail, S, R, stats = rs.schedule(D1, topo, total)
        else:
            off, w, flow, perm = rs.chunk_sort(D1, topo)
            rail, S = rs.lpt_spray(off, w, B, topo, chunkwise=name != "three calls")
            R, stats = rs.eval(off, w, flow, rail, S, B, topo)
        torch.cuda.synchronize()
        n = int(off[-1].item())
        yield name, dict(off=off.cpu().numpy(), w=_u32(w)[:n], flow=_u32(flow)[:n], perm=_u32(perm)[:n],
                         rail=rail.cpu().numpy()[:n], S=S.cpu().numpy(), R=R.cpu().numpy(), stats=stats.cpu().numpy())


def _oracle(D1_np, M, N, C):
    off, w, flow, perm = oracle.chunk_sort_batch(D1_np, M, N, C)
    rail, S = oracle.lpt_batch(off, w, D1_np.shape[0], M, N)
    _, R, stats = oracle.eval_batch(off, w, flow, rail, D1_np.shape[0], M, N)
    return dict(off=off, w=w, flow=flow, perm=perm, rail=rail, S=S, R=R, stats=stats)


def test_single_flow_receive_fixture_end_to_end(golden_dir):
    # Section 4.1 load matrices S and R with the one-to-one rail mapping of the Theorem 3 proof, worked by hand
    g = _read_golden(os.path.join(golden_dir, "single_flow_receive.txt"))
    M, N, C = g["M"][0], g["N"][0], g["C"][0]
    G = M * N
    D1 = np.zeros((1, G, G), dtype=np.int64)
    for d, n, f, m, nbytes in g["flow"]:
        D1[0, d * N + n, f * N + m] = nbytes
    want = _oracle(D1, M, N, C)
    for name, got in _paths(D1, rs.Topo(M, N, C)):
        assert got["off"].tolist() == [0, 6, 6, 6], name
        assert got["w"].tolist() == g["sorted_w"] and got["flow"].tolist() == g["sorted_flow"], name
        assert got["perm"].tolist() == g["perm"] and got["rail"].tolist() == g["rails"], name
        assert got["S"][0, 0].tolist() == g["S0"] and got["S"][0, 1:].tolist() == [[0, 0], [0, 0]], name
        assert got["R"][0].tolist() == [[0, 0], g["R1"], g["R2"]], name
        assert got["stats"][0].tolist() == [g["makespan"][0], 25, 20, g["lower_bound"][0], 47, 10, 6, 3], name
        for key in want:
            assert np.array_equal(got[key], want[key]), (name, key)


def test_graham_tight_fixture_through_the_pipeline(golden_dir):
    # the 4/3 - 1/(3N) family of the Theorem 4 proof: node 0 of a 2 x 3 fabric sends seven flows smaller than a
    # chunk, so its chunk list is exactly the fixture's weights once stage 3 has sorted them
    g = _read_golden(os.path.join(golden_dir, "lpt_graham_tight_n3.txt"))
    N, M, C = g["N"][0], 2, 8
    G = M * N
    D1 = np.zeros((1, G, G), dtype=np.int64)
    cells = [(n, N + m) for n in range(N) for m in range(N)]                # node 0's GPUs -> node 1's GPUs, canonical order
    for (src, dst), wgt in zip(cells, [3, 5, 4, 3, 4, 5, 3]):                # unsorted on purpose: stage 3 orders them
        D1[0, src, dst] = wgt
    want = _oracle(D1, M, N, C)
    for name, got in _paths(D1, rs.Topo(M, N, C)):
        assert got["w"].tolist() == g["weights"], name
        assert got["rail"].tolist() == g["rails"], name
        assert got["S"][0, 0].tolist() == g["loads"] and got["S"][0, 1].tolist() == [0, 0, 0], name
        assert got["stats"][0, 1] == g["lpt_makespan"][0], name             # max send load = LPT makespan of the instance
        assert 3 * N * int(got["stats"][0, 1]) <= (4 * N - 1) * g["opt_makespan"][0], name
        for key in want:
            assert np.array_equal(got[key], want[key]), (name, key)
    # and straight into stage 4, in the given order
    off = torch.tensor([0, 7], dtype=torch.int64, device=DEV)
    w = torch.tensor(g["weights"], dtype=torch.int32, device=DEV)
    for chunkwise in (False, True):
        rail, S = rs.lpt_spray(off, w, 1, rs.Topo(1, N, C), chunkwise=chunkwise)
        assert rail.cpu().tolist() == g["rails"] and S.cpu().view(-1).tolist() == g["loads"]


@pytest.mark.parametrize("M,N,q,B", [(4, 4, 3, 1), (3, 2, 1, 2), (5, 8, 2, 1), (6, 3, 2, 3), (3, 5, 1, 1), (7, 6, 4, 2), (40, 8, 1, 2),
                                     (4, 4, 2, 300)])
def test_uniform_send_gives_uniform_receive(M, N, q, B):
    # Theorem 3 on the all-equal matrix (every entry q*C): every (source GPU, destination node) block is N*q equal chunks in
    # a row, LPT splits it evenly over the rails, and S[k][n] = R[f][n] = (M-1)*N*q*C for all k, f, n; makespan = lower bound
    C = 4096
    D1 = np.repeat(W.symmetric_matrix(M, N, q, C)[None], B, axis=0)
    expect = (M - 1) * N * q * C
    want = _oracle(D1, M, N, C)
    assert np.all(want["S"] == expect) and np.all(want["R"] == expect)
    for name, got in _paths(D1, rs.Topo(M, N, C)):
        assert np.all(got["S"] == expect), name
        assert np.all(got["R"] == expect), name                             # uniform send => uniform receive
        assert np.all(got["stats"][:, 0] == expect) and np.all(got["stats"][:, 3] == expect), name
        assert np.all(got["stats"][:, 7] == 0), name
        assert np.all(got["stats"][:, 6] == M * (M - 1) * N * N * q), name
        for key in want:
            assert np.array_equal(got[key], want[key]), (name, key)
