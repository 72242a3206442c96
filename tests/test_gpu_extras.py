"""GPU parity for the extensions: second all-to-all (transposed traffic) and the arithmetic
comparison schemes.  Bit-exact against the CPU oracle, like everything else."""
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


@pytest.mark.parametrize("M,N,B", [(4, 4, 1), (3, 5, 2), (8, 8, 3), (33, 1, 2), (16, 8, 2), (5, 13, 1)])
def test_transpose_matches_oracle(M, N, B):
    G = M * N
    rng = np.random.default_rng(G + B)
    D1 = rng.integers(0, 1 << 50, size=(B, G, G)).astype(np.int64)
    got = rs.transpose_matrix(torch.from_numpy(D1).to(DEV), rs.Topo(M, N, 4096)).cpu().numpy()
    assert np.array_equal(got, oracle.transpose_batch(D1))


def test_second_all_to_all_pipeline():
    # dispatch and combine of config 1: the combine schedules the transposed matrix; what a node
    # received in the first all-to-all is what it sends in the second
    cfg = W.get_config("c1")
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes)
    logits = W.gen_logits(cfg, 0, device=DEV)
    idx = rs.route_topk(logits, cfg.k)
    D1 = rs.traffic_matrix(idx, 1, cfg.tokens_per_gpu, torch.from_numpy(W.expert_gpu_table(cfg)).to(DEV), cfg.payload_bytes, topo)
    D1T = rs.transpose_matrix(D1, topo)
    res = {}
    for name, D in (("dispatch", D1), ("combine", D1T)):
        off, w, flow, perm = rs.chunk_sort(D, topo)
        rail, S = rs.lpt_spray(off, w, 1, topo)
        R, stats = rs.eval(off, w, flow, rail, S, 1, topo)
        Dh = D.cpu().numpy()
        off_c, w_c, flow_c, perm_c = oracle.chunk_sort_batch(Dh, cfg.M, cfg.N, cfg.chunk_bytes)
        rail_c, S_c = oracle.lpt_batch(off_c, w_c, 1, cfg.M, cfg.N)
        _, R_c, stats_c = oracle.eval_batch(off_c, w_c, flow_c, rail_c, 1, cfg.M, cfg.N)
        n = int(off_c[-1])
        assert np.array_equal(_u32(w)[:n], w_c) and np.array_equal(rail.cpu().numpy()[:n], rail_c)
        assert np.array_equal(S.cpu().numpy(), S_c) and np.array_equal(R.cpu().numpy(), R_c)
        assert np.array_equal(stats.cpu().numpy(), stats_c)
        res[name] = (S_c, R_c)
    assert np.array_equal(res["dispatch"][1].sum(axis=2), res["combine"][0].sum(axis=2))   # received then = sent now
    assert np.array_equal(res["dispatch"][0].sum(axis=2), res["combine"][1].sum(axis=2))


def _records_dev(D1_np, topo):
    D1 = torch.from_numpy(np.ascontiguousarray(D1_np)).to(DEV)
    off, w, flow, perm = rs.chunk_sort(D1, topo, want_perm=False)
    return off, w, flow


def _rand_stack(rng, B, G, C):
    m = rng.integers(0, 6 * C, size=(B, G, G)).astype(np.int64)
    m[rng.random((B, G, G)) < 0.3] = 0
    return m


@pytest.mark.parametrize("policy", ["nic_direct", "flow_hash", "random_spray", "round_robin"])
@pytest.mark.parametrize("M,N,C,B", [(4, 4, 4096, 2), (3, 5, 1000, 3), (8, 8, 65536, 2), (2, 33, 256, 1), (40, 3, 512, 2)])
def test_policy_matches_oracle(policy, M, N, C, B):
    rng = np.random.default_rng(M * 100 + N + B)
    D1 = _rand_stack(rng, B, M * N, C)
    topo = rs.Topo(M, N, C)
    off, w, flow = _records_dev(D1, topo)
    seed = 0xC0FFEE + M
    rail, S = rs.assign_policy(policy, seed, off, w, flow, B, topo)
    R, stats = rs.eval(off, w, flow, rail, S, B, topo)
    n = int(off[-1].item())
    off_h, w_h, flow_h = off.cpu().numpy(), _u32(w)[:n], _u32(flow)[:n]
    rail_c, S_c = oracle.assign_policy(policy, seed, off_h, w_h, flow_h, B, M, N)
    assert np.array_equal(rail.cpu().numpy()[:n], rail_c)
    assert np.array_equal(S.cpu().numpy(), S_c)
    _, R_c, stats_c = oracle.eval_batch(off_h, w_h, flow_h, rail_c, B, M, N)
    assert np.array_equal(R.cpu().numpy(), R_c) and np.array_equal(stats.cpu().numpy(), stats_c)


def test_policy_many_tiny_instances():
    # hundreds of instances inside one streaming tile: most of them go to S through global atomics
    M, N, C, B = 2, 4, 4096, 700
    rng = np.random.default_rng(5)
    D1 = rng.integers(0, 3 * C, size=(B, M * N, M * N)).astype(np.int64)
    D1[rng.random(D1.shape) < 0.8] = 0
    topo = rs.Topo(M, N, C)
    off, w, flow = _records_dev(D1, topo)
    n = int(off[-1].item())
    for policy in ("flow_hash", "round_robin"):
        rail, S = rs.assign_policy(policy, 7, off, w, flow, B, topo)
        rail_c, S_c = oracle.assign_policy(policy, 7, off.cpu().numpy(), _u32(w)[:n], _u32(flow)[:n], B, M, N)
        assert np.array_equal(rail.cpu().numpy()[:n], rail_c) and np.array_equal(S.cpu().numpy(), S_c)


def test_lpt_beats_the_comparison_schemes_on_config2_shape():
    # qualitative statement of Section 6: on skewed MoE traffic the proactive LPT spray is at least as good as
    # static hashing, NIC-direct rails and blind spraying, and sits within a few per cent of the lower bound
    cfg = W.get_config("c2")
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes)
    logits = torch.cat([W.gen_logits(cfg, b, device=DEV) for b in (0, 1)])
    idx = rs.route_topk(logits, cfg.k)
    D1 = rs.traffic_matrix(idx, 2, cfg.tokens_per_gpu, torch.from_numpy(W.expert_gpu_table(cfg)).to(DEV), cfg.payload_bytes, topo)
    off, w, flow, _ = rs.chunk_sort(D1, topo, want_perm=False)
    rail, S = rs.lpt_spray(off, w, 2, topo)
    _, st_lpt = rs.eval(off, w, flow, rail, S, 2, topo)
    st_lpt = st_lpt.cpu().numpy()
    assert np.all(st_lpt[:, 0] <= 1.03 * st_lpt[:, 3])
    for policy in ("nic_direct", "flow_hash", "random_spray", "round_robin"):
        r2, S2 = rs.assign_policy(policy, 1, off, w, flow, 2, topo)
        _, st = rs.eval(off, w, flow, r2, S2, 2, topo)
        st = st.cpu().numpy()
        assert np.all(st[:, 3] == st_lpt[:, 3])                      # same lower bound: same traffic
        assert np.all(st[:, 1] >= st_lpt[:, 1])                      # LPT's worst send NIC is never worse


def test_policy_instances_mostly_empty():
    # thousands of instances of a chunk or two: a streaming tile holds more instance boundaries than it stages in LDS
    M, N, C, B = 2, 2, 4096, 9000
    rng = np.random.default_rng(6)
    D1 = rng.integers(1, 3 * C, size=(B, M * N, M * N)).astype(np.int64)
    D1[rng.random(D1.shape) < 0.93] = 0
    topo = rs.Topo(M, N, C)
    off, w, flow = _records_dev(D1, topo)
    n = int(off[-1].item())
    assert n < 4 * B * M                        # fewer than four chunks per instance on average
    for policy in ("flow_hash", "random_spray", "round_robin", "nic_direct"):
        rail, S = rs.assign_policy(policy, 3, off, w, flow, B, topo)
        rail_c, S_c = oracle.assign_policy(policy, 3, off.cpu().numpy(), _u32(w)[:n], _u32(flow)[:n], B, M, N)
        assert np.array_equal(rail.cpu().numpy()[:n], rail_c) and np.array_equal(S.cpu().numpy(), S_c), policy


def test_policy_and_ports_on_record_arrays_off_16_byte_alignment():
    # records 4 bytes, rails and ports 1 byte past an aligned address: the scalar paths of the comparison schemes
    M, N, C, B, P = 4, 8, 4096, 3, 5
    rng = np.random.default_rng(99)
    D1 = _rand_stack(rng, B, M * N, C)
    topo = rs.Topo(M, N, C)
    off, w0, flow0 = _records_dev(D1, topo)
    n = int(off[-1].item())
    w = torch.empty(n + 8, dtype=torch.int32, device=DEV)[1:n + 1].copy_(w0[:n])
    flow = torch.empty(n + 8, dtype=torch.int32, device=DEV)[1:n + 1].copy_(flow0[:n])
    off_h, w_h, flow_h = off.cpu().numpy(), _u32(w0)[:n], _u32(flow0)[:n]
    for policy in ("nic_direct", "flow_hash", "random_spray", "round_robin"):
        rail = torch.empty(n + 8, dtype=torch.uint8, device=DEV)[1:n + 1]
        S = torch.empty((B, M, N), dtype=torch.int64, device=DEV)
        rs.assign_policy(policy, 11, off, w, flow, B, topo, out=(rail, S))
        rail_c, S_c = oracle.assign_policy(policy, 11, off_h, w_h, flow_h, B, M, N)
        assert np.array_equal(rail.cpu().numpy(), rail_c) and np.array_equal(S.cpu().numpy(), S_c), policy
        port = torch.empty(n + 8, dtype=torch.uint8, device=DEV)[1:n + 1]
        rs.port_round_robin(off, rail, B, topo, P, capacity=n, out=port)
        assert np.array_equal(port.cpu().numpy(), oracle.port_round_robin(off_h, rail_c, B, M, N, P)), policy


@pytest.mark.parametrize("M,N,C,B,P", [(4, 4, 4096, 2, 4), (3, 5, 1000, 3, 3), (8, 8, 65536, 2, 256), (2, 33, 256, 1, 1), (2, 64, 128, 1, 7)])
def test_port_round_robin_matches_oracle(M, N, C, B, P):
    rng = np.random.default_rng(M + N + P)
    D1 = _rand_stack(rng, B, M * N, C)
    topo = rs.Topo(M, N, C)
    off, w, flow = _records_dev(D1, topo)
    rail, S = rs.lpt_spray(off, w, B, topo)
    n = int(off[-1].item())
    port = rs.port_round_robin(off, rail, B, topo, P, capacity=n)
    assert np.array_equal(port.cpu().numpy()[:n], oracle.port_round_robin(off.cpu().numpy(), rail.cpu().numpy()[:n], B, M, N, P))


def test_port_round_robin_long_instances():
    # several tiles per instance, empty instances in between, rails from random spraying
    M, N, C, B, P = 6, 8, 4096, 2, 16
    rng = np.random.default_rng(77)
    G = M * N
    D1 = (np.exp(rng.normal(np.log(60 * C), 1.5, size=(B, G, G))) // 512 * 512).astype(np.int64)
    D1[rng.random((B, G, G)) < 0.5] = 0
    D1[1, 8:16, :] = 0
    topo = rs.Topo(M, N, C)
    off, w, flow = _records_dev(D1, topo)
    n = int(off[-1].item())
    assert np.diff(off.cpu().numpy()).max() > 5 * 4096
    for policy in ("random_spray", "nic_direct"):
        rail, S = rs.assign_policy(policy, 3, off, w, flow, B, topo)
        port = rs.port_round_robin(off, rail, B, topo, P, capacity=n + 1000)
        assert np.array_equal(port.cpu().numpy()[:n], oracle.port_round_robin(off.cpu().numpy(), rail.cpu().numpy()[:n], B, M, N, P))


@pytest.mark.parametrize("fused", [False, True])
def test_whole_path_replays_from_a_hip_graph(fused):
    # the library enqueues kernels only (no allocation, no host synchronisation, no memset nodes), so a caller
    # may capture a pass into a HIP graph; every replay must equal the eager result for the inputs of that moment
    cfg = W.get_config("c2").scaled(batch=2, tokens_per_gpu=4096)
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes)
    B = cfg.batch
    eg = torch.from_numpy(W.expert_gpu_table(cfg)).to(DEV)
    variants = [torch.cat([W.gen_logits(cfg, b + 10 * v, device=DEV) for b in range(B)]) for v in range(3)]
    logits = variants[0].clone()
    rows = logits.shape[0]
    cap = 0
    for v in variants:                                              # capacity that fits every variant
        D = rs.traffic_matrix(rs.route_topk(v, cfg.k), B, cfg.tokens_per_gpu, eg, cfg.payload_bytes, topo)
        cap = max(cap, int(rs.chunk_count(D, topo)[-1].item()))
    plan = rs.Plan(topo, B, cap, DEV, rows=rows, k=cfg.k)

    ws_rt = torch.empty(rs.route_traffic_workspace_bytes(B, cfg.tokens_per_gpu, cfg.E, cfg.k, topo), dtype=torch.uint8, device=DEV)

    def step(eager=False):
        if fused and not eager:                                     # the two fused calls, checked against the five stages
            rs.route_traffic(logits, cfg.k, B, cfg.tokens_per_gpu, eg, cfg.payload_bytes, topo, out=(plan.topk_idx, plan.D1), ws=ws_rt)
            plan.schedule_one_call()
        else:
            plan.route(logits, cfg.tokens_per_gpu, eg, cfg.payload_bytes)
            plan.schedule()

    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rnd in range(5):
        logits.copy_(variants[rnd % 3])
        step(eager=True)                                            # eager reference for these inputs
        torch.cuda.synchronize()
        want = [t.clone() for t in (plan.topk_idx, plan.D1, plan.chunk_off, plan.S, plan.R, plan.stats)]
        n = int(plan.chunk_off[-1].item())
        want_rec = [t[:n].clone() for t in (plan.chunk_w, plan.chunk_flow, plan.perm, plan.rail)]
        for t in (plan.topk_idx, plan.D1, plan.chunk_off, plan.S, plan.R, plan.stats, plan.chunk_w, plan.chunk_flow, plan.perm, plan.rail):
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = (plan.topk_idx, plan.D1, plan.chunk_off, plan.S, plan.R, plan.stats)
        assert all(torch.equal(a, b) for a, b in zip(want, got)), f"replay {rnd}"
        got_rec = (plan.chunk_w, plan.chunk_flow, plan.perm, plan.rail)
        assert all(torch.equal(a, b[:n]) for a, b in zip(want_rec, got_rec)), f"replay {rnd} records"
