"""GPU parity at the full sizes of the five workloads, in the launch shapes the benchmark uses.

Where the oracle can afford it everything is compared element by element (c1 elsewhere, c2 here);
for the large configurations chunk_off is compared in full, a seeded sample of whole instances and of
whole matrices is compared element by element, and properties that hold at any size are checked over
all outputs on the device: byte and rail conservation, rail range, descending order inside every
instance, makespan >= lower bound, max-min send load <= w_max.
"""
import gc

import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

rs = pytest.importorskip("paper_2510_19262_amd")
DEV = "cuda:0"


def _free():
    gc.collect()
    torch.cuda.empty_cache()


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _schedule_dev(D1, topo, want_perm=True):
    batch = D1.shape[0]
    off, w, flow, perm = rs.chunk_sort(D1, topo, want_perm=want_perm)
    rail, S = rs.lpt_spray(off, w, batch, topo)
    R, stats = rs.eval(off, w, flow, rail, S, batch, topo)
    torch.cuda.synchronize()
    return dict(off=off, w=w, flow=flow, perm=perm, rail=rail, S=S, R=R, stats=stats)


def _check_one_call(g, D1, topo):
    """railsched_schedule on the same input: every output equal to the three calls' (which the oracle checks)."""
    total = int(g["off"][-1].item())
    off, w, flow, perm, rail, S, R, stats = rs.schedule(D1, topo, total, want_perm=g["perm"] is not None)
    torch.cuda.synchronize()
    assert torch.equal(off, g["off"]) and torch.equal(S, g["S"]) and torch.equal(R, g["R"]) and torch.equal(stats, g["stats"])
    assert torch.equal(w[:total], g["w"][:total]) and torch.equal(flow[:total], g["flow"][:total])
    assert torch.equal(rail[:total], g["rail"][:total])
    if perm is not None:
        assert torch.equal(perm[:total], g["perm"][:total])


def _check_instances(g, D1_host_of, M, N, C, insts):
    """Whole instances against the oracle: records, permutation, rails, send loads."""
    off = g["off"].cpu().numpy()
    for inst in insts:
        print(f"  instance {inst}: {int(off[inst + 1] - off[inst])} chunks against the oracle", flush=True)
        b, k = divmod(int(inst), M)
        cw, cf = oracle.chunk_split(D1_host_of(b), M, N, C, k)
        sw, sf, sp = oracle.sort_desc(cw, cf)
        rail_c, L = oracle.lpt(sw, N)
        o, e = int(off[inst]), int(off[inst + 1])
        assert e - o == sw.size, f"instance {inst}: {e - o} chunks vs {sw.size}"
        assert np.array_equal(_u32(g["w"][o:e]), sw), f"instance {inst}: chunk_w"
        assert np.array_equal(_u32(g["flow"][o:e]), sf), f"instance {inst}: chunk_flow"
        if g["perm"] is not None:
            assert np.array_equal(_u32(g["perm"][o:e]), sp), f"instance {inst}: perm"
        assert np.array_equal(g["rail"][o:e].cpu().numpy(), rail_c), f"instance {inst}: rail"
        assert np.array_equal(g["S"].view(-1, N)[inst].cpu().numpy(), L), f"instance {inst}: S"


def _check_matrices(g, D1_host_of, M, N, C, mats):
    """Whole matrices against the oracle: R and stats (needs every instance of the matrix)."""
    for b in mats:
        D = np.ascontiguousarray(D1_host_of(b))[None]
        off_c, w_c, flow_c, _ = oracle.chunk_sort_batch(D, M, N, C, want_perm=False)
        rail_c, S_c = oracle.lpt_batch(off_c, w_c, 1, M, N)
        _, R_c, stats_c = oracle.eval_batch(off_c, w_c, flow_c, rail_c, 1, M, N)
        assert np.array_equal(g["S"][b].cpu().numpy(), S_c[0]), f"matrix {b}: S"
        assert np.array_equal(g["R"][b].cpu().numpy(), R_c[0]), f"matrix {b}: R"
        assert np.array_equal(g["stats"][b].cpu().numpy(), stats_c[0]), f"matrix {b}: stats"


def _check_properties(g, D1, M, N):
    """Properties that hold at any size, evaluated on the device over every output."""
    B = D1.shape[0]
    G = M * N
    total = int(g["off"][-1].item())
    S, R, stats = g["S"], g["R"], g["stats"]
    # inter-node bytes of every source node / destination node
    blocks = D1.view(B, M, N, M, N).sum(dim=(2, 4))                        # D2[b][k][f]
    inter = blocks - torch.diag_embed(torch.diagonal(blocks, dim1=1, dim2=2))
    assert torch.equal(S.sum(dim=2), inter.sum(dim=2))                      # sum_n S[k][n] = sum_{f!=k} D2[k][f]
    assert torch.equal(R.sum(dim=2), inter.sum(dim=1))                      # sum_n R[f][n] = sum_{k!=f} D2[k][f]
    assert torch.equal(S.sum(dim=1), R.sum(dim=1))                          # what leaves on rail n arrives on rail n
    assert torch.equal(stats[:, 0], torch.maximum(S.amax(dim=(1, 2)), R.amax(dim=(1, 2))))
    assert torch.equal(stats[:, 4], inter.sum(dim=(1, 2)))
    assert bool((stats[:, 0] >= stats[:, 3]).all())                         # makespan >= lower bound
    assert bool((stats[:, 7] <= stats[:, 5]).all())                         # greedy: max-min send load <= w_max
    assert torch.equal(stats[:, 6], g["off"][M::M] - g["off"][:-1:M])
    if total:
        assert int(g["rail"][:total].max().item()) < N
        # weights never increase inside an instance: an increase may only sit on an instance boundary
        w = g["w"][:total]
        step = 1 << 28
        starts = g["off"][:-1]
        for lo in range(0, total - 1, step):
            hi = min(lo + step, total - 1)
            up = torch.nonzero(w[lo + 1:hi + 1] > w[lo:hi]).view(-1) + (lo + 1)
            if up.numel():
                assert bool(torch.isin(up, starts).all()), "weights increase inside an instance"
        assert int(g["flow"][:total].max().item()) < N * G


# ---------------------------------------------------------------------------------------- c2
@pytest.mark.timeout(900)
def test_c2_full_every_array():
    cfg = W.get_config("c2")
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes, cfg.rail_bw_Bps)
    B = cfg.batch
    logits = torch.cat([W.gen_logits(cfg, b, device=DEV) for b in range(B)])
    eg_np = W.expert_gpu_table(cfg)
    eg = torch.from_numpy(eg_np).to(DEV)
    idx = rs.route_topk(logits, cfg.k)
    D1 = rs.traffic_matrix(idx, B, cfg.tokens_per_gpu, eg, cfg.payload_bytes, topo)
    g = _schedule_dev(D1, topo)

    idx_c = oracle.route_topk(logits.cpu().numpy(), cfg.k)
    assert np.array_equal(idx.cpu().numpy(), idx_c)
    D1_c = oracle.traffic_matrix(idx_c, B, cfg.tokens_per_gpu, eg_np, cfg.payload_bytes, cfg.M, cfg.N)
    assert np.array_equal(D1.cpu().numpy(), D1_c)
    off_c, w_c, flow_c, perm_c = oracle.chunk_sort_batch(D1_c, cfg.M, cfg.N, cfg.chunk_bytes)
    rail_c, S_c = oracle.lpt_batch(off_c, w_c, B, cfg.M, cfg.N)
    _, R_c, stats_c = oracle.eval_batch(off_c, w_c, flow_c, rail_c, B, cfg.M, cfg.N)
    n = int(off_c[-1])
    assert np.array_equal(g["off"].cpu().numpy(), off_c)
    assert np.array_equal(_u32(g["w"])[:n], w_c) and np.array_equal(_u32(g["flow"])[:n], flow_c)
    assert np.array_equal(_u32(g["perm"])[:n], perm_c)
    assert np.array_equal(g["rail"].cpu().numpy()[:n], rail_c)
    assert np.array_equal(g["S"].cpu().numpy(), S_c) and np.array_equal(g["R"].cpu().numpy(), R_c)
    assert np.array_equal(g["stats"].cpu().numpy(), stats_c)
    _check_properties(g, D1, cfg.M, cfg.N)

    # the same batch through the two fused calls, in the launch configuration the benchmark times
    idx2, D12 = rs.route_traffic(logits, cfg.k, B, cfg.tokens_per_gpu, eg, cfg.payload_bytes, topo)
    assert torch.equal(idx2, idx) and torch.equal(D12, D1)
    off2, w2, flow2, perm2, rail2, S2, R2, stats2 = rs.schedule(D12, topo, n)
    assert np.array_equal(off2.cpu().numpy(), off_c)
    assert np.array_equal(_u32(w2)[:n], w_c) and np.array_equal(_u32(flow2)[:n], flow_c) and np.array_equal(_u32(perm2)[:n], perm_c)
    assert np.array_equal(rail2.cpu().numpy()[:n], rail_c)
    assert np.array_equal(S2.cpu().numpy(), S_c) and np.array_equal(R2.cpu().numpy(), R_c)
    assert np.array_equal(stats2.cpu().numpy(), stats_c)
    del logits, idx, D1, g, idx2, D12
    _free()


# ---------------------------------------------------------------------------------------- c3
@pytest.mark.timeout(900)
def test_c3_full_batch_sampled():
    cfg = W.get_config("c3")
    M, N, C, B = cfg.M, cfg.N, cfg.chunk_bytes, cfg.batch
    topo = rs.Topo(M, N, C)
    D1 = W.gen_flow_matrices_device(cfg, DEV)                              # 1024 matrices of 256x256, 512 MiB
    g = _schedule_dev(D1, topo)
    _check_one_call(g, D1, topo)
    D1_h = D1.cpu().numpy()
    assert np.array_equal(g["off"].cpu().numpy(), oracle.chunk_count_batch(D1_h, M, N, C))
    total = int(g["off"][-1].item())
    assert total > 3_000_000_000                                           # ~3.85e9 chunks in flight
    sizes = np.diff(g["off"].cpu().numpy())
    rng = np.random.default_rng(3)
    insts = set(rng.integers(0, B * M, size=20).tolist()) | {0, B * M - 1, int(sizes.argmax()), int(sizes.argmin())}
    _check_instances(g, lambda b: D1_h[b], M, N, C, sorted(insts))
    _check_matrices(g, lambda b: D1_h[b], M, N, C, [0, 517, B - 1])
    _check_properties(g, D1, M, N)
    del D1, g
    _free()


# ---------------------------------------------------------------------------------------- c4
@pytest.mark.timeout(900)
def test_c4_all_layers_sampled():
    cfg = W.get_config("c4")
    M, N, C, B = cfg.M, cfg.N, cfg.chunk_bytes, cfg.batch
    topo = rs.Topo(M, N, C, cfg.rail_bw_Bps)
    eg_np = W.expert_gpu_table(cfg)
    eg = torch.from_numpy(eg_np).to(DEV)
    rows = cfg.rows_per_layer                                               # 4 194 304 rows x 256 experts = 4 GiB per layer
    D1 = torch.empty((B, cfg.G, cfg.G), dtype=torch.int64, device=DEV)
    rng = np.random.default_rng(4)
    checked_layers = {0, 37}
    for b in range(B):                                                      # the 244 GiB of logits stream through layer by layer
        logits = W.gen_logits(cfg, b, device=DEV)
        idx = rs.route_topk(logits, cfg.k)
        rs.traffic_matrix(idx, 1, cfg.tokens_per_gpu, eg, cfg.payload_bytes, topo, out=D1[b:b + 1])
        # sampled rows of every layer against the oracle (plus whole slabs of two layers)
        pick = np.sort(rng.choice(rows, size=4096, replace=False))
        pick_t = torch.from_numpy(pick).to(DEV)
        assert np.array_equal(idx[pick_t].cpu().numpy(), oracle.route_topk(logits[pick_t].cpu().numpy(), cfg.k)), f"layer {b}"
        if b in checked_layers:
            slab = slice(1_000_000, 1_300_000)
            assert np.array_equal(idx[slab].cpu().numpy(), oracle.route_topk(logits[slab].cpu().numpy(), cfg.k))
            D1_c = oracle.traffic_matrix(idx.cpu().numpy(), 1, cfg.tokens_per_gpu, eg_np, cfg.payload_bytes, M, N)
            assert np.array_equal(D1[b].cpu().numpy(), D1_c[0]), f"layer {b}: D1"
        del logits, idx
    per_gpu = cfg.tokens_per_gpu * cfg.k * cfg.payload_bytes
    assert bool((D1.sum(dim=2) == per_gpu).all())                           # every source GPU routes the same bytes
    g = _schedule_dev(D1, topo)
    _check_one_call(g, D1, topo)
    D1_h = D1.cpu().numpy()
    assert np.array_equal(g["off"].cpu().numpy(), oracle.chunk_count_batch(D1_h, M, N, C))
    sizes = np.diff(g["off"].cpu().numpy())
    insts = set(rng.integers(0, B * M, size=24).tolist()) | {0, B * M - 1, int(sizes.argmax()), int(sizes.argmin())}
    _check_instances(g, lambda b: D1_h[b], M, N, C, sorted(insts))
    _check_matrices(g, lambda b: D1_h[b], M, N, C, [0, 37, B - 1])
    _check_properties(g, D1, M, N)
    del D1, g
    _free()


# ---------------------------------------------------------------------------------------- c5
C5_MATRICES = (0, 3, 128, 255)          # of the 256 the workload has; each is ~3.9e9 chunks and runs on its own
C5_WHOLE_MATRICES = (3, 255)           # these also meet the oracle in full: S, R and stats of all 128 instances


@pytest.mark.timeout(900)
@pytest.mark.parametrize("b", C5_MATRICES)
def test_c5_matrix(b):
    cfg = W.get_config("c5")
    M, N, C = cfg.M, cfg.N, cfg.chunk_bytes
    topo = rs.Topo(M, N, C)
    D1 = W.gen_flow_matrices_device(cfg, DEV, first=b, count=1)             # one 1024x1024 matrix: ~4e9 chunks
    g = _schedule_dev(D1, topo, want_perm=False)
    _check_one_call(g, D1, topo)
    D1_h = D1.cpu().numpy()
    off_g = g["off"].cpu().numpy()
    assert np.array_equal(off_g, oracle.chunk_count_batch(D1_h, M, N, C))
    sizes = np.diff(off_g)
    assert sizes.max() > 10_000_000
    order = np.argsort(sizes)
    # the largest instance (the heavy tail this workload exists for), the smallest and the median, element by element
    _check_instances(g, lambda _: D1_h[0], M, N, C, [int(order[-1]), int(order[0]), int(order[len(order) // 2])])
    _check_properties(g, D1, M, N)
    if b in C5_WHOLE_MATRICES:
        # every instance of the matrix through the oracle, one node at a time (its records would not fit otherwise)
        off_c, S_c, R_c, stats_c = oracle.schedule_matrix_by_node(D1_h[0], M, N, C)
        assert np.array_equal(off_g, off_c)
        assert np.array_equal(g["S"][0].cpu().numpy(), S_c), "S"
        assert np.array_equal(g["R"][0].cpu().numpy(), R_c), "R"
        assert np.array_equal(g["stats"][0].cpu().numpy(), stats_c), "stats"
    del D1, g
    _free()


def test_c5_small_matrices_elementwise():
    # the stress topology (128 nodes x 8 rails, 16 KiB chunks) with flows 1000x smaller, all arrays
    cfg = W.get_config("c5").scaled(mu_bytes=16 * 1024)
    M, N, C = cfg.M, cfg.N, cfg.chunk_bytes
    D1 = W.gen_flow_matrices(cfg, first=0, count=2)
    g = _schedule_dev(torch.from_numpy(D1).to(DEV), rs.Topo(M, N, C))
    off_c, w_c, flow_c, perm_c = oracle.chunk_sort_batch(D1, M, N, C)
    rail_c, S_c = oracle.lpt_batch(off_c, w_c, 2, M, N)
    _, R_c, stats_c = oracle.eval_batch(off_c, w_c, flow_c, rail_c, 2, M, N)
    n = int(off_c[-1])
    assert np.array_equal(g["off"].cpu().numpy(), off_c)
    assert np.array_equal(_u32(g["w"])[:n], w_c) and np.array_equal(_u32(g["flow"])[:n], flow_c)
    assert np.array_equal(_u32(g["perm"])[:n], perm_c) and np.array_equal(g["rail"].cpu().numpy()[:n], rail_c)
    assert np.array_equal(g["S"].cpu().numpy(), S_c) and np.array_equal(g["R"].cpu().numpy(), R_c)
    assert np.array_equal(g["stats"].cpu().numpy(), stats_c)
