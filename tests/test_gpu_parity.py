"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, bit for bit.

All outputs are integers, so every comparison is exact equality.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

rs = pytest.importorskip("paper_2510_19262_amd")
DEV = "cuda:0"


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def gpu_schedule(D1_np, topo, want_perm=True):
    """Stages 3-5 on the GPU for a [batch][G][G] matrix stack; everything back as numpy."""
    D1 = torch.from_numpy(np.ascontiguousarray(D1_np)).to(DEV)
    batch = D1.shape[0]
    off, w, flow, perm = rs.chunk_sort(D1, topo, want_perm=want_perm)
    rail, S = rs.lpt_spray(off, w, batch, topo)
    R, stats = rs.eval(off, w, flow, rail, S, batch, topo)
    torch.cuda.synchronize()
    total = int(off[-1].item())
    return dict(off=off.cpu().numpy(), w=_u32(w)[:total], flow=_u32(flow)[:total],
                perm=None if perm is None else _u32(perm)[:total], rail=rail.cpu().numpy()[:total],
                S=S.cpu().numpy(), R=R.cpu().numpy(), stats=stats.cpu().numpy())


def gpu_schedule_one_call(D1_np, topo, want_perm=True, capacity=None):
    """Stages 3-5 through railsched_schedule."""
    D1 = torch.from_numpy(np.ascontiguousarray(D1_np)).to(DEV)
    if capacity is None:
        capacity = int(rs.chunk_count(D1, topo)[-1].item())
    off, w, flow, perm, rail, S, R, stats = rs.schedule(D1, topo, capacity, want_perm=want_perm)
    torch.cuda.synchronize()
    total = int(off[-1].item())
    return dict(off=off.cpu().numpy(), w=_u32(w)[:total], flow=_u32(flow)[:total],
                perm=None if perm is None else _u32(perm)[:total], rail=rail.cpu().numpy()[:total],
                S=S.cpu().numpy(), R=R.cpu().numpy(), stats=stats.cpu().numpy())


def cpu_schedule(D1_np, M, N, C, intra=0):
    D1_np = np.ascontiguousarray(D1_np, dtype=np.int64)
    B = D1_np.shape[0]
    off, w, flow, perm = oracle.chunk_sort_batch(D1_np, M, N, C, intra)
    rail, S = oracle.lpt_batch(off, w, B, M, N)
    Ssum, R, stats = oracle.eval_batch(off, w, flow, rail, B, M, N)
    assert np.array_equal(S, Ssum)
    return dict(off=off, w=w, flow=flow, perm=perm, rail=rail, S=S, R=R, stats=stats)


def assert_same(g, c, what=""):
    for key in ("off", "w", "flow", "perm", "rail", "S", "R", "stats"):
        if g[key] is None:
            continue
        assert g[key].shape == c[key].shape, f"{what}{key}: shape {g[key].shape} vs {c[key].shape}"
        if not np.array_equal(g[key], c[key]):
            bad = np.flatnonzero(g[key].reshape(-1) != c[key].reshape(-1))
            raise AssertionError(f"{what}{key}: {bad.size} mismatches, first at {bad[:5]}: "
                                 f"gpu {g[key].reshape(-1)[bad[:5]]} cpu {c[key].reshape(-1)[bad[:5]]}")


# ------------------------------------------------------------------------------ stage 1
@pytest.mark.parametrize("E,k,rows", [(8, 2, 100_003), (8, 1, 777), (8, 8, 513), (4, 2, 1000), (3, 2, 1001), (5, 3, 999),
                                      (16, 4, 2049), (12, 5, 300), (32, 2, 1025), (64, 6, 700), (100, 7, 333),
                                      (128, 8, 511), (256, 8, 4099), (250, 9, 130), (512, 4, 129), (1000, 3, 65),
                                      (1024, 16, 70), (1, 1, 50), (8, 2, 1), (256, 8, 1)])
def test_topk_matches_oracle(E, k, rows):
    rng = np.random.default_rng(E * 1000 + k)
    x = rng.standard_normal((rows, E)).astype(np.float32)
    x[rows // 2:] = np.round(x[rows // 2:] * 2) / 2          # half the rows: few distinct values, many ties
    got = rs.route_topk(torch.from_numpy(x).to(DEV), k).cpu().numpy()
    assert np.array_equal(got, oracle.route_topk(x, k))


def test_topk_crafted_ties():
    rows = [[1.25] * 8, [0, 5, 1, 5, 5, -1, 2, 0], [-1, -0.0, 0.0, -2, 0.0, -0.0, -3, -4], [3, 3, 2, 2, 1, 1, 0, 0],
            [-5, -5, -5, -5, -5, -5, -5, -4]]
    x = np.array(rows, dtype=np.float32)
    for k in (1, 2, 4, 8):
        got = rs.route_topk(torch.from_numpy(x).to(DEV), k).cpu().numpy()
        assert np.array_equal(got, oracle.route_topk(x, k))
    x = np.zeros((130, 256), dtype=np.float32)                 # all equal across 64 lanes: first k indices
    got = rs.route_topk(torch.from_numpy(x).to(DEV), 8).cpu().numpy()
    assert np.array_equal(got, np.tile(np.arange(8), (130, 1)))


@pytest.mark.parametrize("E,k", [(64, 6), (128, 8), (256, 8), (256, 64), (200, 5), (36, 16)])
def test_topk_values_that_differ_in_the_last_bits(E, k):
    # logits packed so closely that only the lowest mantissa bits (or nothing) separate the leaders
    rng = np.random.default_rng(E + k)
    rows = 1500
    base = rng.choice(np.array([1.0, -1.0, 3.5, -0.0, 1e-30, -7e5], dtype=np.float32), size=(rows, 1))
    ulps = rng.integers(0, 6, size=(rows, E)).astype(np.int32)
    x = (base.view(np.int32) + ulps).view(np.float32)
    x[::3] = rng.standard_normal((x[::3].shape[0], E)).astype(np.float32)     # ordinary rows in the same wavefronts
    assert np.all(np.isfinite(x))
    got = rs.route_topk(torch.from_numpy(x).to(DEV), k).cpu().numpy()
    assert np.array_equal(got, oracle.route_topk(x, k))


@pytest.mark.parametrize("E,k,rows", [(64, 8, 3000), (96, 3, 1111), (128, 8, 2000), (256, 8, 1500), (256, 1, 700), (40, 8, 900)])
def test_topk_rows_full_of_exact_ties(E, k, rows):
    # logits on a lattice of 13 values: every row has many equal logits, among the winners and at the cut
    rng = np.random.default_rng(E * 7 + k)
    x = (rng.integers(-6, 7, size=(rows, E)) * 0.25).astype(np.float32)
    x[::7] = 0.0                                                     # whole rows of one value
    x[1::7, ::2] = -0.0
    got = rs.route_topk(torch.from_numpy(x).to(DEV), k).cpu().numpy()
    assert np.array_equal(got, oracle.route_topk(x, k))


@pytest.mark.parametrize("E,k", [(64, 8), (128, 5), (256, 8), (8, 2), (200, 8)])
def test_topk_denormals_and_signed_zeros(E, k):
    # denormal logits of both signs, +0 and -0 (which tie), tiny normals: order must be the IEEE one
    rng = np.random.default_rng(E + 3 * k)
    rows = 2000
    pool = np.array([0.0, -0.0, 1e-45, -1e-45, 3e-39, -3e-39, 1.1754944e-38, -1.1754944e-38, 1e-30, -1e-30, 2e-45, -2e-45],
                    dtype=np.float32)
    x = rng.choice(pool, size=(rows, E)).astype(np.float32)
    got = rs.route_topk(torch.from_numpy(x).to(DEV), k).cpu().numpy()
    assert np.array_equal(got, oracle.route_topk(x, k))


def test_topk_unaligned_rows_and_empty():
    x = torch.randn(1001 * 8 + 1, device=DEV)[1:].view(1001, 8)   # base pointer off 16-byte alignment
    assert np.array_equal(rs.route_topk(x.contiguous(), 2).cpu().numpy(), oracle.route_topk(x.cpu().numpy(), 2))
    empty = torch.empty((0, 8), device=DEV)
    assert rs.route_topk(empty, 2).shape == (0, 2)


def test_logit_generator_is_device_independent():
    cfg = W.get_config("c2")
    a = W.gen_logits(cfg, 3, device="cpu", rows=50_000)
    b = W.gen_logits(cfg, 3, device=DEV, rows=50_000).cpu()
    assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    c = W.gen_logits(cfg, 3, device=DEV, row_start=1000, rows=10).cpu()
    assert torch.equal(a[1000:1010].view(torch.int32), c.view(torch.int32))


# ------------------------------------------------------------------------------ stage 2
@pytest.mark.parametrize("M,N,E,k,R,tok,batch", [(4, 4, 8, 2, 2, 2048, 1), (2, 3, 6, 3, 1, 777, 2), (3, 2, 7, 2, 3, 1000, 3),
                                                 (8, 8, 8, 2, 8, 4096, 2), (1, 1, 4, 1, 1, 10, 1), (2, 2, 4, 4, 2, 70001, 1),
                                                 (16, 8, 256, 8, 1, 300, 1), (2, 2, 16, 4, 1000, 2100, 1), (3, 2, 9, 2, 1200, 1500, 2)])
def test_traffic_matrix_matches_oracle(M, N, E, k, R, tok, batch):
    rng = np.random.default_rng(M * 100 + N * 10 + E)
    G = M * N
    eg = rng.integers(0, G, size=(E, R)).astype(np.int32)
    rows = batch * G * tok
    idx = np.argsort(rng.random((rows, E)), axis=1)[:, :k].astype(np.int32)
    topo = rs.Topo(M, N, 4096)
    got = rs.traffic_matrix(torch.from_numpy(idx).to(DEV), batch, tok, torch.from_numpy(eg).to(DEV), 2048, topo)
    assert np.array_equal(got.cpu().numpy(), oracle.traffic_matrix(idx, batch, tok, eg, 2048, M, N))


def test_traffic_matrix_skewed_bins():
    # every token picks expert 0 first: all hits of a source GPU land in one bin
    M, N, E, k, tok = 2, 4, 8, 2, 50_000
    G = M * N
    eg = np.arange(E, dtype=np.int32).reshape(E, 1)
    idx = np.tile(np.array([[0, 1]], dtype=np.int32), (G * tok, 1))
    got = rs.traffic_matrix(torch.from_numpy(idx).to(DEV), 1, tok, torch.from_numpy(eg).to(DEV), 8192, rs.Topo(M, N, 4096))
    assert np.array_equal(got.cpu().numpy(), oracle.traffic_matrix(idx, 1, tok, eg, 8192, M, N))


# ------------------------------------------------------------------------------ stages 1+2 in one call
def _coarse_logits(rng, rows, E):
    # a coarse lattice: exact ties between logits of a row are common
    return (rng.integers(-6, 7, size=(rows, E)) * 0.25).astype(np.float32)


@pytest.mark.parametrize("M,N,E,k,R,tok,batch,want_idx", [
    (4, 4, 8, 2, 2, 2048, 1, True), (8, 8, 8, 2, 8, 4096, 2, True), (8, 8, 8, 2, 8, 4096, 2, False),
    (2, 3, 6, 3, 1, 777, 2, True), (3, 2, 7, 2, 3, 5000, 3, True), (1, 1, 4, 1, 1, 10, 1, True),
    (2, 2, 4, 4, 2, 70001, 1, True), (2, 2, 3, 2, 5, 2049, 2, True), (2, 2, 8, 8, 4, 3000, 1, True),
    (2, 4, 1, 1, 1, 100, 1, True), (2, 4, 2, 1, 2, 4097, 1, False), (2, 2, 5, 5, 2, 0, 2, True),
    (4, 2, 16, 4, 2, 1000, 2, True), (2, 2, 64, 8, 1, 300, 1, True),
    (2, 2, 8, 2, 1500, 3001, 1, True), (2, 3, 7, 3, 2000, 2500, 2, True)])     # placement tables too large for LDS
def test_route_traffic_matches_the_two_stages_of_the_oracle(M, N, E, k, R, tok, batch, want_idx):
    rng = np.random.default_rng(M * 1000 + N * 100 + E * 10 + k)
    G = M * N
    eg = rng.integers(0, G, size=(E, R)).astype(np.int32)
    rows = batch * G * tok
    x = _coarse_logits(rng, rows, E)
    topo = rs.Topo(M, N, 4096)
    idx, D1 = rs.route_traffic(torch.from_numpy(x).to(DEV).view(rows, E), k, batch, tok, torch.from_numpy(eg).to(DEV), 2048, topo,
                               want_idx=want_idx)
    want = oracle.route_topk(x, k) if rows else np.empty((0, k), np.int32)
    if want_idx:
        assert np.array_equal(idx.cpu().numpy(), want)
    else:
        assert idx is None
    assert np.array_equal(D1.cpu().numpy(), oracle.traffic_matrix(want, batch, tok, eg, 2048, M, N))


@pytest.mark.parametrize("M,N,E,k,R,tok,batch,kind", [
    (4, 4, 256, 8, 2, 700, 1, "normal"), (8, 8, 256, 8, 4, 1031, 2, "normal"), (2, 3, 128, 8, 3, 513, 2, "normal"),
    (2, 2, 64, 6, 1, 2000, 1, "normal"), (2, 2, 40, 8, 5, 333, 3, "normal"), (3, 2, 200, 5, 2, 129, 2, "normal"),
    (2, 2, 256, 1, 2, 257, 1, "normal"), (2, 2, 96, 3, 7, 31, 2, "normal"), (4, 4, 256, 8, 2, 300, 1, "lattice"),
    (2, 2, 128, 4, 2, 300, 2, "lattice"), (2, 2, 64, 8, 3, 100, 1, "lattice"), (2, 2, 256, 8, 1, 64, 1, "bunched"),
    (64, 8, 256, 8, 4, 40, 1, "normal"), (2, 2, 256, 8, 2048, 600, 1, "normal")])
def test_route_traffic_wide_rows_with_and_without_indices(M, N, E, k, R, tok, batch, kind):
    # rows of 33..256 logits with k <= 8: with the indices the two stages run back to back, without them gating and traffic
    # matrix come out of one pass over the logits.  Token counts that are no multiple of a workgroup's share, replica counts
    # that are no power of two, a placement table too large for LDS, logits full of exact ties (every wavefront takes the
    # exact path) and winners bunched in one lane's experts.
    rng = np.random.default_rng(M * 1000 + N * 100 + E * 10 + k + R)
    G = M * N
    eg = rng.integers(0, G, size=(E, R)).astype(np.int32)
    rows = batch * G * tok
    if kind == "lattice":
        x = _coarse_logits(rng, rows, E)
    else:
        x = rng.standard_normal((rows, E)).astype(np.float32)
        if kind == "bunched":
            x[:, :4] += 9.0
            x[:, 32:36] += 8.0                                      # experts 0-3 and 32-35 sit in the same lane of the row
    topo = rs.Topo(M, N, 4096)
    want = oracle.route_topk(x, k)
    D1_want = oracle.traffic_matrix(want, batch, tok, eg, 1536, M, N)
    xd, egd = torch.from_numpy(x).to(DEV).view(rows, E), torch.from_numpy(eg).to(DEV)
    for want_idx in (True, False):
        idx, D1 = rs.route_traffic(xd, k, batch, tok, egd, 1536, topo, want_idx=want_idx)
        if want_idx:
            assert np.array_equal(idx.cpu().numpy(), want)
        else:
            assert idx is None
        assert np.array_equal(D1.cpu().numpy(), D1_want), f"D1, want_idx={want_idx}"


def test_route_traffic_unaligned_logits_and_stale_output():
    M, N, E, k, R, tok = 2, 2, 8, 2, 2, 3001
    rng = np.random.default_rng(5)
    G = M * N
    rows = G * tok
    x = _coarse_logits(rng, rows, E)
    eg = rng.integers(0, G, size=(E, R)).astype(np.int32)
    buf = torch.zeros(rows * E + 1, device=DEV)
    buf[1:] = torch.from_numpy(x).to(DEV).view(-1)
    lg = buf[1:].view(rows, E)                                   # base pointer off 16-byte alignment
    D1 = torch.full((1, G, G), -7, dtype=torch.int64, device=DEV)   # stale contents must be overwritten
    idx = torch.full((rows, k), -1, dtype=torch.int32, device=DEV)
    rs.route_traffic(lg, k, 1, tok, torch.from_numpy(eg).to(DEV), 512, rs.Topo(M, N, 4096), out=(idx, D1))
    want = oracle.route_topk(x, k)
    assert np.array_equal(idx.cpu().numpy(), want)
    assert np.array_equal(D1.cpu().numpy(), oracle.traffic_matrix(want, 1, tok, eg, 512, M, N))


def test_route_traffic_wide_rows_need_the_index_array():
    topo = rs.Topo(2, 2, 4096)
    lg = torch.zeros((4 * 8, 16), device=DEV)
    eg = torch.zeros((16, 1), dtype=torch.int32, device=DEV)
    with pytest.raises(rs.RailschedError):
        rs.route_traffic(lg, 2, 1, 8, eg, 64, topo, want_idx=False)


# ------------------------------------------------------------------------------ stages 3-5
def _rand_stack(rng, B, G, C, p_zero=0.3, hi=6):
    m = rng.integers(0, hi * C, size=(B, G, G)).astype(np.int64)
    m[rng.random((B, G, G)) < p_zero] = 0
    m[rng.random((B, G, G)) < 0.2] //= C
    m[rng.random((B, G, G)) < 0.2] = 3 * C
    return m


# ------------------------------------------------------------------------------ stages 3-5 in one call
@pytest.mark.parametrize("M,N,C,B,intra,perm", [
    (4, 4, 65536, 1, 0, True), (3, 2, 100, 4, 0, True), (3, 2, 100, 4, 1, True), (5, 3, 1000, 3, 0, False),
    (2, 8, 4096, 5, 0, True), (8, 8, 262144, 3, 0, True), (6, 5, 12345, 2, 0, True), (2, 16, 64, 2, 0, True),
    (3, 20, 512, 2, 0, False), (2, 32, 256, 1, 0, True), (1, 4, 64, 2, 1, True), (7, 1, 64, 3, 0, True),
    (4, 4, 1, 1, 0, True), (16, 8, 4096, 2, 0, True), (8, 8, 262144, 32, 0, True), (2, 2, 7, 300, 0, True)])
def test_schedule_one_call_matches_oracle(M, N, C, B, intra, perm):
    rng = np.random.default_rng(M * 1000 + N * 10 + B + 5)
    hi = 6 if C > 1 else 40
    D1 = _rand_stack(rng, B, M * N, C, hi=hi)
    topo = rs.Topo(M, N, C, include_intra_node=intra)
    g = gpu_schedule_one_call(D1, topo, want_perm=perm)
    c = cpu_schedule(D1, M, N, C, intra)
    if not perm:
        c["perm"] = None
    assert_same(g, c)


def test_schedule_one_call_degenerate_instances():
    # instances with no chunks at all, with tails only, with full chunks only, and with fewer full chunks than rails
    M, N, C = 3, 4, 1000
    G = M * N
    D1 = np.zeros((5, G, G), dtype=np.int64)
    D1[1, :, :] = 999                        # tails only
    D1[2, :, :] = 3000                       # full chunks only
    D1[3, 0, 5] = 2000; D1[3, 1, 9] = 1      # two full chunks (< N) and one tail in node 0, nothing elsewhere
    D1[4, 4, 0] = 123456                     # one flow
    topo = rs.Topo(M, N, C)
    assert_same(gpu_schedule_one_call(D1, topo), cpu_schedule(D1, M, N, C))


def test_schedule_one_call_large_batches_take_the_three_stages():
    # more instances than the one-workgroup-per-instance shape accepts, and a generous capacity
    rng = np.random.default_rng(77)
    M, N, C, B = 4, 2, 512, 400              # 1600 instances
    D1 = _rand_stack(rng, B, M * N, C)
    topo = rs.Topo(M, N, C)
    assert_same(gpu_schedule_one_call(D1, topo), cpu_schedule(D1, M, N, C))
    D1b = _rand_stack(rng, 2, M * N, C)
    total = int(oracle.chunk_count_batch(D1b, M, N, C)[-1])
    assert_same(gpu_schedule_one_call(D1b, topo, capacity=total + 12345), cpu_schedule(D1b, M, N, C))


@pytest.mark.parametrize("M,N,C,B,intra,perm", [(40, 8, 4096, 2, 0, True), (3, 40, 512, 2, 0, True), (4, 4, 64, 300, 0, False),
                                               (2, 64, 128, 1, 0, True), (6, 5, 12345, 200, 1, True), (2, 2, 1 << 31, 3, 0, True)])
def test_schedule_one_call_three_stage_shapes(M, N, C, B, intra, perm):
    # shapes outside the one-workgroup-per-instance limits: many instances, many flows per instance, huge chunks
    rng = np.random.default_rng(M * 1000 + N * 10 + B + 9)
    D1 = _rand_stack(rng, B, M * N, min(C, 1 << 20), hi=9)
    if C > 1 << 30:
        D1 = D1 * 5000                                           # bytes of the order of the chunk size
    topo = rs.Topo(M, N, C, include_intra_node=intra)
    g = gpu_schedule_one_call(D1, topo, want_perm=perm)
    c = cpu_schedule(D1, M, N, C, intra)
    if not perm:
        c["perm"] = None
    assert_same(g, c)


def test_schedule_one_call_capacity_overflow_leaves_records_alone():
    rng = np.random.default_rng(78)
    M, N, C, B = 4, 4, 4096, 2
    D1n = _rand_stack(rng, B, M * N, C)
    D1 = torch.from_numpy(D1n).to(DEV)
    topo = rs.Topo(M, N, C)
    total = int(oracle.chunk_count_batch(D1n, M, N, C)[-1])
    cap = total - 1
    out = (torch.empty(B * M + 1, dtype=torch.int64, device=DEV), torch.full((cap,), -1, dtype=torch.int32, device=DEV),
           torch.full((cap,), -1, dtype=torch.int32, device=DEV), None, torch.full((cap,), 255, dtype=torch.uint8, device=DEV),
           torch.empty((B, M, N), dtype=torch.int64, device=DEV), torch.empty((B, M, N), dtype=torch.int64, device=DEV),
           torch.empty((B, 8), dtype=torch.int64, device=DEV))
    rs.schedule(D1, topo, cap, out=out)
    torch.cuda.synchronize()
    assert int(out[0][-1].item()) == total
    assert bool((out[1] == -1).all()) and bool((out[2] == -1).all()) and bool((out[4] == 255).all())
    assert all(bool((t == -1).all()) for t in out[5:])                  # S, R, stats say so without a read-back of chunk_off
    with pytest.raises(rs.RailschedError) as err:                       # and the synchronising call reports it to the host
        rs.check_capacity(out[0], B, topo, cap)
    assert err.value.status == -4 and err.value.total == total
    assert rs.check_capacity(out[0], B, topo, total) == total
    # the same through the three-stage shape (more instances than one workgroup each serves)
    B2 = 300
    D2n = _rand_stack(rng, B2, M * N, C)
    total2 = int(oracle.chunk_count_batch(D2n, M, N, C)[-1])
    cap2 = total2 - 1
    out2 = (torch.empty(B2 * M + 1, dtype=torch.int64, device=DEV), torch.full((cap2,), -1, dtype=torch.int32, device=DEV),
            torch.full((cap2,), -1, dtype=torch.int32, device=DEV), None, torch.full((cap2,), 255, dtype=torch.uint8, device=DEV),
            torch.empty((B2, M, N), dtype=torch.int64, device=DEV), torch.empty((B2, M, N), dtype=torch.int64, device=DEV),
            torch.empty((B2, 8), dtype=torch.int64, device=DEV))
    rs.schedule(torch.from_numpy(D2n).to(DEV), topo, cap2, out=out2)
    torch.cuda.synchronize()
    assert int(out2[0][-1].item()) == total2
    assert bool((out2[1] == -1).all()) and bool((out2[2] == -1).all()) and bool((out2[4] == 255).all())
    assert all(bool((t == -1).all()) for t in out2[5:])


@pytest.mark.parametrize("B", [2, 300, 8200])      # wide shape of stage 4, and packed shape (N = 4: from 32768 instances on)
@pytest.mark.parametrize("chunkwise", [False, True])
def test_three_calls_capacity_overflow_touches_no_record(B, chunkwise):
    # stage 3 finds more chunks than the arrays hold: stages 4 and 5, given the same capacity, must neither read nor
    # write a record and must mark their outputs (sentinel-filled arrays sized exactly `capacity` stay as they were)
    rng = np.random.default_rng(79 + B)
    M, N, C = 4, 4, 4096
    D1n = _rand_stack(rng, B, M * N, C)
    topo = rs.Topo(M, N, C)
    total = int(oracle.chunk_count_batch(D1n, M, N, C)[-1])
    cap = total - 1
    off = torch.empty(B * M + 1, dtype=torch.int64, device=DEV)
    w = torch.full((cap,), -1, dtype=torch.int32, device=DEV)
    flow = torch.full((cap,), -1, dtype=torch.int32, device=DEV)
    perm = torch.full((cap,), -1, dtype=torch.int32, device=DEV)
    rail = torch.full((cap,), 255, dtype=torch.uint8, device=DEV)
    port = torch.full((cap,), 254, dtype=torch.uint8, device=DEV)
    S = torch.zeros((B, M, N), dtype=torch.int64, device=DEV)
    R = torch.zeros((B, M, N), dtype=torch.int64, device=DEV)
    stats = torch.zeros((B, 8), dtype=torch.int64, device=DEV)
    rs.chunk_sort(torch.from_numpy(D1n).to(DEV), topo, capacity=cap, out=(off, w, flow, perm))
    rs.lpt_spray(off, w, B, topo, out=(rail, S), chunkwise=chunkwise, capacity=cap)
    rs.eval(off, w, flow, rail, S, B, topo, out=(R, stats), capacity=cap)
    rs.port_round_robin(off, rail, B, topo, 4, capacity=cap, out=port)
    torch.cuda.synchronize()
    assert int(off[-1].item()) == total
    assert bool((w == -1).all()) and bool((flow == -1).all()) and bool((perm == -1).all())
    assert bool((rail == 255).all()) and bool((port == 254).all())
    assert bool((S == -1).all()) and bool((R == -1).all()) and bool((stats == -1).all())
    for policy in ("nic_direct", "random_spray"):
        S.zero_()
        rs.assign_policy(policy, 5, off, w, flow, B, topo, out=(rail, S), capacity=cap)
        torch.cuda.synchronize()
        assert bool((rail == 255).all()) and bool((S == -1).all())
    # with room for every chunk the same buffers come out as the oracle says (one spare record stays untouched)
    cap = total + 1
    w, flow, perm = (torch.full((cap,), -1, dtype=torch.int32, device=DEV) for _ in range(3))
    rail = torch.full((cap,), 255, dtype=torch.uint8, device=DEV)
    rs.chunk_sort(torch.from_numpy(D1n).to(DEV), topo, capacity=cap, out=(off, w, flow, perm))
    rs.lpt_spray(off, w, B, topo, out=(rail, S), chunkwise=chunkwise, capacity=cap)
    rs.eval(off, w, flow, rail, S, B, topo, out=(R, stats), capacity=cap)
    torch.cuda.synchronize()
    c = cpu_schedule(D1n, M, N, C)
    assert np.array_equal(_u32(w)[:total], c["w"]) and np.array_equal(rail.cpu().numpy()[:total], c["rail"])
    assert np.array_equal(S.cpu().numpy(), c["S"]) and np.array_equal(R.cpu().numpy(), c["R"]) and np.array_equal(stats.cpu().numpy(), c["stats"])
    assert int(w[-1].item()) == -1 and int(rail[-1].item()) == 255


@pytest.mark.parametrize("M,N,C,B,intra", [(4, 4, 65536, 1, 0), (3, 2, 100, 4, 0), (3, 2, 100, 4, 1), (5, 3, 1000, 3, 0),
                                           (2, 8, 4096, 5, 0), (8, 8, 262144, 3, 0), (6, 5, 12345, 2, 0), (2, 16, 64, 2, 0),
                                           (3, 20, 512, 2, 0), (2, 33, 256, 1, 0), (2, 64, 128, 1, 0), (1, 4, 64, 2, 1),
                                           (7, 1, 64, 3, 0), (4, 4, 1, 1, 0), (40, 8, 4096, 2, 0)])
def test_schedule_matches_oracle(M, N, C, B, intra):
    rng = np.random.default_rng(M * 1000 + N * 10 + B)
    hi = 6 if C > 1 else 40
    D1 = _rand_stack(rng, B, M * N, C, hi=hi)
    topo = rs.Topo(M, N, C, include_intra_node=intra)
    assert_same(gpu_schedule(D1, topo), cpu_schedule(D1, M, N, C, intra))


def test_schedule_long_instances_and_empty_ones():
    # heavy-tailed flows: instances from zero to tens of thousands of chunks, several fill tiles per instance
    M, N, C, B = 6, 8, 4096, 3
    rng = np.random.default_rng(42)
    G = M * N
    D1 = (np.exp(rng.normal(np.log(40 * C), 2.0, size=(B, G, G))) // 512 * 512).astype(np.int64)
    D1[rng.random((B, G, G)) < 0.6] = 0
    D1[0, 8:16, :] = 0                      # node 1 of matrix 0 sends nothing
    D1[2] = 0                               # a whole empty matrix
    topo = rs.Topo(M, N, C)
    g, c = gpu_schedule(D1, topo), cpu_schedule(D1, M, N, C)
    assert np.diff(c["off"]).max() > 3 * 16384
    assert_same(g, c)


def test_schedule_without_perm_and_all_zero():
    M, N, C = 3, 4, 1024
    rng = np.random.default_rng(5)
    D1 = _rand_stack(rng, 2, M * N, C)
    g = gpu_schedule(D1, rs.Topo(M, N, C), want_perm=False)
    assert g["perm"] is None
    assert_same(g, cpu_schedule(D1, M, N, C))
    Z = np.zeros((2, M * N, M * N), dtype=np.int64)
    assert_same(gpu_schedule(Z, rs.Topo(M, N, C)), cpu_schedule(Z, M, N, C))


def test_chunk_sort_capacity_guard():
    M, N, C = 3, 4, 1024
    rng = np.random.default_rng(6)
    D1 = torch.from_numpy(_rand_stack(rng, 2, M * N, C)).to(DEV)
    topo = rs.Topo(M, N, C)
    total = int(rs.chunk_count(D1, topo)[-1].item())
    sentinel = 0x5A5A5A5A
    out = (torch.empty(2 * M + 1, dtype=torch.int64, device=DEV),
           torch.full((total,), sentinel, dtype=torch.int32, device=DEV),
           torch.full((total,), sentinel, dtype=torch.int32, device=DEV),
           torch.full((total,), sentinel, dtype=torch.int32, device=DEV))
    off, w, flow, perm = rs.chunk_sort(D1, topo, capacity=total - 1, out=out)
    torch.cuda.synchronize()
    assert int(off[-1].item()) == total                               # offsets are complete ...
    assert bool((w == sentinel).all()) and bool((flow == sentinel).all()) and bool((perm == sentinel).all())  # ... records untouched
    off, w, flow, perm = rs.chunk_sort(D1, topo, capacity=total, out=out)
    torch.cuda.synchronize()
    assert not bool((w == sentinel).any())


# ------------------------------------------------------------------------------ stage 4 alone
def _lpt_case(weights_per_inst, M, N, batch=1):
    """Arbitrary per-instance weight lists straight into stage 4."""
    lens = [len(w) for w in weights_per_inst]
    assert len(lens) == batch * M
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    w = np.concatenate([np.asarray(x, dtype=np.uint32) for x in weights_per_inst]) if sum(lens) else np.zeros(0, np.uint32)
    topo = rs.Topo(M, N, 1 << 20)
    wt = torch.from_numpy(w.view(np.int32).copy()).to(DEV) if w.size else torch.zeros(1, dtype=torch.int32, device=DEV)
    rail_c, S_c = oracle.lpt_batch(off, w, batch, M, N)
    for chunkwise, ws in ((False, "auto"), (True, "auto"), (True, None)):      # with the optional workspace and without
        rail, S = rs.lpt_spray(torch.from_numpy(off).to(DEV), wt, batch, topo, chunkwise=chunkwise, ws=ws)
        assert np.array_equal(rail.cpu().numpy()[:w.size], rail_c), f"rail, chunkwise={chunkwise}, ws={ws}"
        assert np.array_equal(S.cpu().numpy(), S_c), f"S, chunkwise={chunkwise}, ws={ws}"


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 8, 11, 16, 24, 32, 40, 64])
def test_lpt_random_weights_any_order(N):
    rng = np.random.default_rng(N)
    M = 19
    insts = []
    for i in range(M):
        n = int(rng.integers(0, 700))
        w = rng.integers(0, 1 << 18, size=n)
        if i % 3 == 0:
            w = np.sort(w)[::-1]
        if i % 5 == 0 and n:
            w[:] = w[0]                                           # one long run of equal weights
        insts.append(w)
    _lpt_case(insts, M, N)


@pytest.mark.parametrize("N", [2, 8, 16, 64])
def test_lpt_large_weights_take_the_exact_path(N):
    rng = np.random.default_rng(100 + N)
    M = 9
    insts = []
    for i in range(M):
        n = int(rng.integers(1, 300))
        w = rng.integers(0, 1 << 32, size=n, dtype=np.uint64)
        if i % 2:                                                 # small weights first, a huge one mid-stream
            w = rng.integers(0, 1 << 16, size=n, dtype=np.uint64)
            w[n // 2] = (1 << 32) - 1
        insts.append(w.astype(np.uint32))
    _lpt_case(insts, M, N)


def test_lpt_weights_at_the_packing_limit():
    # weights just below / at / above the switch-over, many chunks so the loads pass 2^32
    for N, lim in ((8, ((0xFFFFFFFF >> 3) // 34) - 1), (8, ((0xFFFFFFFF >> 3) // 66) - 1), (64, ((0xFFFFFFFF >> 6) // 66) - 1),
                   (4, ((0xFFFFFFFF >> 2) // 66) - 1), (16, ((0xFFFFFFFF >> 4) // 66) - 1),
                   (1, ((0xFFFFFFFF >> 2) // 66) - 1), (2, ((0xFFFFFFFF >> 2) // 66) - 1), (5, ((0xFFFFFFFF >> 3) // 66) - 1)):
        insts = [np.full(400, lim, dtype=np.uint32), np.full(400, lim + 1, dtype=np.uint32),
                 np.concatenate([np.full(200, lim), np.arange(200, 0, -1)]).astype(np.uint32)]
        _lpt_case(insts, 3, N)


def test_lpt_tight_family_and_small_cases():
    _lpt_case([[5, 5, 4, 4, 3, 3, 3]], 1, 3)
    _lpt_case([[9, 7, 3], [], [4]], 3, 5)
    _lpt_case([[], []], 2, 8)
    _lpt_case([[7] * 1000], 1, 8)


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 6, 7, 8, 12, 16, 31, 32, 48, 64])
def test_lpt_long_runs_of_equal_weights(N):
    # runs much longer than a period, entered from balanced and from unbalanced loads, of every
    # residue modulo N, with weights that make max-min equal to, just below and just above the run weight
    rng = np.random.default_rng(500 + N)
    insts = []
    for i in range(23):
        parts = []
        for _ in range(int(rng.integers(1, 6))):
            w = int(rng.choice([0, 1, 7, 4096, 65536, 262144, 100000]))
            parts.append(np.full(int(rng.integers(1, 400)), w))
            if rng.random() < 0.5:
                parts.append(rng.integers(0, 300000, size=int(rng.integers(0, 40))))
        w = np.concatenate(parts)
        if i % 2 == 0:
            w = np.sort(w)[::-1]
        insts.append(w)
    insts.append(np.concatenate([[300], np.full(500, 300)]))                 # spread == weight on entry
    insts.append(np.concatenate([[299], np.full(500, 300)]))
    insts.append(np.concatenate([[301], np.full(500, 300)]))
    insts.append(np.concatenate([[1000, 900, 800], np.full(777, 100), np.full(333, 3)]))
    _lpt_case(insts, len(insts), N)


def test_lpt_chunk_lists_from_stage3_shapes():
    # what stage 3 emits: one long run of C, then sorted tails on a coarse lattice
    rng = np.random.default_rng(77)
    C, gran = 262144, 8192
    insts = []
    for i in range(40):
        nfull = int(rng.integers(0, 9000))
        tails = np.sort(rng.integers(1, C // gran, size=int(rng.integers(0, 450))) * gran)[::-1]
        insts.append(np.concatenate([np.full(nfull, C), tails]))
    _lpt_case(insts, 8, 8, batch=5)


def _many_instances_case(N, n_inst, per_wave, period, seed):
    """Ragged lengths, runs, mixed weights, one instance that drags its wavefront onto the exact path, and weights at, one
    above and around the packing limit (periods of `period` chunks), in wavefronts of their own (`per_wave` instances each),
    with loads that pass 2^32."""
    gw = 4 if N <= 4 else 8 if N <= 8 else 16 if N <= 16 else 32
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, 120, size=n_inst)
    lens[rng.random(n_inst) < 0.02] = 0
    lens[:50] = rng.integers(300, 900, size=50)
    insts = []
    for i, n in enumerate(lens):
        kind = i % 4
        if kind == 0:
            w = np.full(n, 65536)
        elif kind == 1:
            w = np.sort(rng.integers(1, 32, size=n) * 8192)[::-1]
        elif kind == 2:
            w = np.concatenate([np.full(n // 2, 262144), np.sort(rng.integers(1, 262144, size=n - n // 2))[::-1]])
        else:
            w = rng.integers(0, 1 << 20, size=n)
        insts.append(w)
    insts[7] = np.concatenate([[5_000_000_00], rng.integers(0, 1 << 30, size=40)])   # drags its wavefront onto the exact path
    lim = ((0xFFFFFFFF >> (gw.bit_length() - 1)) // (period + 2)) - 1
    insts[20 * per_wave] = np.full(700, lim)
    insts[30 * per_wave + 1] = np.full(700, lim + 1)
    insts[40 * per_wave] = np.concatenate([np.full(300, lim), np.arange(300, 0, -1)])
    insts[50 * per_wave] = np.concatenate([np.full(130, lim), [lim + 1], np.full(130, lim - 1)])   # leaves the packed keys mid-way
    insts[60 * per_wave + 2] = np.concatenate([np.full(1000, 4096), np.full(333, 4095), np.full(200, 7)])   # long closed-form runs
    _lpt_case(insts, 1, N, batch=n_inst)                      # one node per matrix, n_inst matrices


@pytest.mark.parametrize("N", [1, 2, 3, 4, 7, 8, 20, 32])
def test_lpt_packed_shape_many_instances(N):
    # enough instances that the packed shape is taken: several share a wavefront, one per lane group
    gw = 4 if N <= 4 else 8 if N <= 8 else 32
    n_inst = (2048 * (64 // gw) if gw < 32 else 5200) + 37
    _many_instances_case(N, n_inst, 64 // gw, 32 if gw == 4 else 64, 900 + N)


@pytest.mark.parametrize("N,n_inst", [(1, 1100), (3, 4133), (4, 2500), (5, 4133), (8, 4133), (8, 16000), (11, 1400), (13, 8229), (16, 8229),
                                      (16, 20000)])
def test_lpt_rows_shape_many_instances(N, n_inst):
    # four instances per wavefront, one per row of 16 lanes: the shape between the wide and the packed one (N <= 16)
    _many_instances_case(N, n_inst, 4, 64, 1900 + N)


def test_lpt_many_instances():
    rng = np.random.default_rng(9)
    M, batch = 37, 11
    insts = [np.sort(rng.integers(1, 1 << 16, size=int(rng.integers(0, 200))))[::-1] for _ in range(M * batch)]
    _lpt_case(insts, M, 8, batch)


@pytest.mark.parametrize("N", [4, 8])
def test_lpt_instances_mostly_empty(N):
    # tens of thousands of instances of 0-2 chunks: a streaming tile of the leading-run kernel holds more instance
    # boundaries than it stages in LDS and reads them from memory instead
    rng = np.random.default_rng(77 + N)
    n_inst = 60000
    lens = rng.choice([0, 0, 0, 0, 0, 1, 2], size=n_inst)                 # 0.43 chunks per instance: 2 400 instances per 1 Ki tile
    insts = [np.sort(rng.integers(1, 9, size=n) * 4096)[::-1] for n in lens]
    _lpt_case(insts, 1, N, batch=n_inst)


# ------------------------------------------------------------------------------ whole path on the paper-shaped configs
def _moe_pipeline_gpu(cfg, layers):
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes, cfg.rail_bw_Bps)
    logits = torch.cat([W.gen_logits(cfg, b, device=DEV) for b in layers])
    eg = torch.from_numpy(W.expert_gpu_table(cfg)).to(DEV)
    idx = rs.route_topk(logits, cfg.k)
    D1 = rs.traffic_matrix(idx, len(layers), cfg.tokens_per_gpu, eg, cfg.payload_bytes, topo)
    torch.cuda.synchronize()
    return logits, idx, D1, topo


def test_config1_end_to_end():
    cfg = W.get_config("c1")
    logits, idx, D1, topo = _moe_pipeline_gpu(cfg, [0])
    x = logits.cpu().numpy()
    idx_c = oracle.route_topk(x, cfg.k)
    assert np.array_equal(idx.cpu().numpy(), idx_c)
    D1_c = oracle.traffic_matrix(idx_c, 1, cfg.tokens_per_gpu, W.expert_gpu_table(cfg), cfg.payload_bytes, cfg.M, cfg.N)
    assert np.array_equal(D1.cpu().numpy(), D1_c)
    g, c = gpu_schedule(D1_c, topo), cpu_schedule(D1_c, cfg.M, cfg.N, cfg.chunk_bytes)
    assert_same(g, c, "c1 ")
    assert c["stats"][0, 0] >= c["stats"][0, 3]


def test_config2_two_layers_elementwise():
    cfg = W.get_config("c2")
    logits, idx, D1, topo = _moe_pipeline_gpu(cfg, [0, 31])
    idx_c = oracle.route_topk(logits.cpu().numpy(), cfg.k)
    assert np.array_equal(idx.cpu().numpy(), idx_c)
    D1_c = oracle.traffic_matrix(idx_c, 2, cfg.tokens_per_gpu, W.expert_gpu_table(cfg), cfg.payload_bytes, cfg.M, cfg.N)
    assert np.array_equal(D1.cpu().numpy(), D1_c)
    assert_same(gpu_schedule(D1_c, topo), cpu_schedule(D1_c, cfg.M, cfg.N, cfg.chunk_bytes), "c2 ")


def test_config3_shape_small_batch():
    cfg = W.get_config("c3")
    D1 = W.gen_flow_matrices(cfg, first=0, count=2)
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes)
    assert_same(gpu_schedule(D1, topo), cpu_schedule(D1, cfg.M, cfg.N, cfg.chunk_bytes), "c3 ")


def test_config4_shape_reduced_tokens():
    # DeepSeek-V3-shaped routing (E=256, top-8, 512 GPUs, 2 experts/GPU, 4 replicas) with 256 tokens per GPU
    cfg = W.get_config("c4").scaled(tokens_per_gpu=256)
    logits, idx, D1, topo = _moe_pipeline_gpu(cfg, [0])
    idx_c = oracle.route_topk(logits.cpu().numpy(), cfg.k)
    assert np.array_equal(idx.cpu().numpy(), idx_c)
    D1_c = oracle.traffic_matrix(idx_c, 1, cfg.tokens_per_gpu, W.expert_gpu_table(cfg), cfg.payload_bytes, cfg.M, cfg.N)
    assert np.array_equal(D1.cpu().numpy(), D1_c)
    assert_same(gpu_schedule(D1_c, topo), cpu_schedule(D1_c, cfg.M, cfg.N, cfg.chunk_bytes), "c4 ")


# ------------------------------------------------------------------------------ record arrays off their natural alignment
@pytest.mark.parametrize("skew", [1, 4, 68])
@pytest.mark.parametrize("M,N,C,B", [(4, 4, 4096, 2), (8, 8, 262144, 3), (4, 2, 512, 400), (3, 20, 512, 2)])
def test_record_arrays_off_16_byte_alignment(M, N, C, B, skew):
    # chunk_w / chunk_flow / perm start 4 bytes, rail 1 byte past an aligned address (the scalar paths of every kernel),
    # or 16 / 272 bytes past one (vector paths whose kilobytes do not sit on the boundaries the kernels cut their steps at)
    rng = np.random.default_rng(M * 31 + N * 7 + B)
    D1n = _rand_stack(rng, B, M * N, C)
    c = cpu_schedule(D1n, M, N, C)
    n = int(c["off"][-1])
    topo = rs.Topo(M, N, C)
    D1 = torch.from_numpy(D1n).to(DEV)

    def bufs():
        w = torch.empty(n + 80, dtype=torch.int32, device=DEV)[skew:n + skew]
        flow = torch.empty(n + 80, dtype=torch.int32, device=DEV)[skew:n + skew]
        perm = torch.empty(n + 80, dtype=torch.int32, device=DEV)[skew:n + skew]
        rail = torch.empty(n + 80, dtype=torch.uint8, device=DEV)[skew:n + skew]
        return w, flow, perm, rail

    def same(off, w, flow, perm, rail, S, R, stats, what):
        g = dict(off=off.cpu().numpy(), w=_u32(w)[:n], flow=_u32(flow)[:n], perm=_u32(perm)[:n], rail=rail.cpu().numpy()[:n],
                 S=S.cpu().numpy(), R=R.cpu().numpy(), stats=stats.cpu().numpy())
        assert_same(g, c, what)

    w, flow, perm, rail = bufs()
    off = torch.empty(B * M + 1, dtype=torch.int64, device=DEV)
    S = torch.empty((B, M, N), dtype=torch.int64, device=DEV)
    rs.chunk_sort(D1, topo, capacity=n, out=(off, w, flow, perm))
    rs.lpt_spray(off, w, B, topo, out=(rail, S))
    R, stats = rs.eval(off, w, flow, rail, S, B, topo)
    same(off, w, flow, perm, rail, S, R, stats, "three calls")

    w, flow, perm, rail = bufs()
    out = (torch.empty(B * M + 1, dtype=torch.int64, device=DEV), w, flow, perm, rail, torch.empty_like(S), torch.empty_like(S),
           torch.empty((B, 8), dtype=torch.int64, device=DEV))
    rs.schedule(D1, topo, n, out=out)
    same(*out, "one call")
