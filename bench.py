#!/usr/bin/env python3
"""Benchmark of the whole rail-spraying path on one MI355X (default: the c2 workload; --config picks another).

A step is one pass of all five stages (route_topk -> traffic_matrix -> chunk_sort -> lpt_spray ->
eval) over one batch of the Mixtral-8x7B-shaped workload, through two calls: railsched_route_traffic
(stages 1-2 in one pass over the logits) and railsched_schedule (stages 3-5, one workgroup per
instance).  Both write the same bytes as the separate calls - asserted here on every output array;
the same step through the five separate calls is timed too and reported as "staged", and the
throughput with two steps in flight on two streams as "two_steps_in_flight".  Workload: 8 nodes x
8 rails, 8 experts top-2, 16384 tokens per GPU, 8 KiB tokens, 256 KiB chunks, 32 layers = 32
traffic matrices of 64x64.
Inputs (1 GiB of fp32 router logits, synthetic, seeded) are resident in HBM before timing starts.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes the launches of one route_traffic call (main kernel + reduction of the slice counts) move on this
# workload, from rocprofv3 FETCH_SIZE / WRITE_SIZE scaled by a 1 GiB copy of known traffic (profiles/c2_whole_path.md).
# route_traffic_kernel 1043.54 MiB read + 272.00 MiB written, rt_reduce_kernel 16.04 MiB read + 1.00 MiB written.
ROUTE_TRAFFIC_C2_TRAFFIC_BYTES = int((1043.54 + 272.00 + 16.04 + 1.00) * 1024 * 1024)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c2",
                    help="workload: c2 (default, the benchmark workload) or c1 = whole path with resident logits; c4 = whole path, "
                         "logits streamed layer by layer; c3, c5 = stages 3-5 on synthetic flow matrices")
    ap.add_argument("--matrices", type=int, default=0,
                    help="c3/c5: matrices per step (0 = all of c3, one of c5: a c5 matrix alone is 3.9e9 chunks)")
    ap.add_argument("--cpu-layers", type=int, default=-1,
                    help="layers of the workload the CPU oracle is timed on (-1 = all, 0 = skip)")
    ap.add_argument("--skip-extras", action="store_true",
                    help="only the two timed regions (fused and staged step): no supplementary measurements; used for profiles, "
                         "so that a kernel's average duration is that of the timed region")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device copy first: a kernel of known traffic to scale profiler byte counters by")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the rails and the other GPUs are simulated "
              "arithmetically); --gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as W
    import paper_2510_19262_amd as rs

    rs.load()                                       # fails loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = W.get_config(args.config)
    if cfg.kind == "flows":
        return bench_flows(cfg, args, rs, W, torch, np)
    if cfg.rows_per_layer * cfg.batch * cfg.E * 4 > 64 << 30:
        return bench_streamed(cfg, args, rs, W, torch, np)
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes, cfg.rail_bw_Bps)
    B, G = cfg.batch, cfg.G
    rows = B * cfg.rows_per_layer

    # ---- inputs, resident in HBM
    logits = torch.empty((rows, cfg.E), dtype=torch.float32, device=dev)
    for b in range(B):
        logits[b * cfg.rows_per_layer:(b + 1) * cfg.rows_per_layer] = W.gen_logits(cfg, b, device=dev)
    eg_np = W.expert_gpu_table(cfg)
    expert_gpu = torch.from_numpy(eg_np).to(dev)

    if args.copy_probe:
        probe = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        probe.copy_(logits.view(-1)[: 1 << 28])
        torch.cuda.synchronize()
        del probe

    # ---- size the record arrays once (count query), then a plan that allocates nothing per step
    idx0 = rs.route_topk(logits, cfg.k)
    D10 = rs.traffic_matrix(idx0, B, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo)
    total_chunks = int(rs.chunk_count(D10, topo)[-1].item())
    del idx0, D10
    plan = rs.Plan(topo, B, total_chunks, dev, rows=rows, k=cfg.k, want_perm=True)

    ws_rt = torch.empty(max(rs.route_traffic_workspace_bytes(B, cfg.tokens_per_gpu, cfg.E, cfg.k, topo), 256), dtype=torch.uint8, device=dev)
    names = {True: ("route_traffic", "schedule"),
             False: ("route_topk", "traffic_matrix", "chunk_sort", "lpt_spray", "eval")}

    def step(fused, events=None):
        marks = []
        def mark():
            if events is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                marks.append(e)
        mark()
        if fused:
            rs.route_traffic(logits, cfg.k, B, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo,
                             out=(plan.topk_idx, plan.D1), ws=ws_rt); mark()
        else:
            rs.route_topk(logits, cfg.k, out=plan.topk_idx); mark()
            rs.traffic_matrix(plan.topk_idx, B, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo, out=plan.D1); mark()
        if fused:
            plan.schedule_one_call(); mark()
        else:
            rs.chunk_sort(plan.D1, topo, capacity=plan.capacity,
                          out=(plan.chunk_off, plan.chunk_w, plan.chunk_flow, plan.perm), ws=plan.ws_sort); mark()
            rs.lpt_spray(plan.chunk_off, plan.chunk_w, B, topo, out=(plan.rail, plan.S)); mark()
            rs.eval(plan.chunk_off, plan.chunk_w, plan.chunk_flow, plan.rail, plan.S, B, topo,
                    out=(plan.R, plan.stats), ws=plan.ws_eval); mark()
        if events is not None:
            events.append(marks)

    def run(fused):
        for _ in range(args.warmup):
            step(fused)
        torch.cuda.synchronize()
        ev = []
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(fused, ev)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms = {n: 0.0 for n in names[fused]}
        for marks in ev:
            for i, n in enumerate(names[fused]):
                ms[n] += marks[i].elapsed_time(marks[i + 1])
        return (t1 - t0) * 1e3 / args.steps, {n: v / args.steps for n, v in ms.items()}

    staged_ms_per_step, staged_ms = run(False)
    keep = ("topk_idx", "D1", "chunk_off", "chunk_w", "chunk_flow", "perm", "rail", "S", "R", "stats")
    staged_out = {n: getattr(plan, n).clone() for n in keep}
    for n in keep[2:]:
        getattr(plan, n).fill_(0)
    ms_per_step, stage_ms = run(True)                # the timed region the headline value comes from
    for n in keep:                                   # both ways give the same bytes
        m = total_chunks if n in ("chunk_w", "chunk_flow", "perm", "rail") else None
        assert torch.equal(staged_out[n][:m], getattr(plan, n)[:m]), n
    del staged_out

    assert int(plan.chunk_off[-1].item()) == total_chunks

    piped_ms = chunkwise_ms = graph_ms = None
    schemes = combine = sweep = placement = None
    stats = plan.stats.cpu().numpy()
    ratio = stats[:, 0] / np.maximum(stats[:, 3], 1)
    if not args.skip_extras:
        # ---- supplementary: throughput with two steps in flight (two streams of default priority, outputs double-buffered):
        # the latency-bound stages 3-5 of one step run beside the bandwidth-bound stages 1-2 of the next
        plan_b = rs.Plan(topo, B, total_chunks, dev, rows=rows, k=cfg.k, want_perm=True)
        ws_rt_b = torch.empty_like(ws_rt)
        lanes = ((plan, ws_rt, torch.cuda.Stream()), (plan_b, ws_rt_b, torch.cuda.Stream()))

        def piped(i):
            p, w, s_ = lanes[i % 2]
            with torch.cuda.stream(s_):
                rs.route_traffic(logits, cfg.k, B, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo, out=(p.topk_idx, p.D1), ws=w)
                p.schedule_one_call()
        for i in range(2 * max(args.warmup, 1)):
            piped(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(2 * args.steps):
            piped(i)
        torch.cuda.synchronize()
        piped_ms = (time.perf_counter() - t0) * 1e3 / (2 * args.steps)
        assert torch.equal(plan_b.stats, plan.stats) and torch.equal(plan_b.rail, plan.rail) and torch.equal(plan_b.R, plan.R)
        del plan_b, ws_rt_b

        # ---- supplementary: the same step replayed from a HIP graph (the library enqueues kernels only: no allocation,
        # no host synchronisation, no memset nodes), which takes the host's launch calls out of the step
        want_g = [t.clone() for t in (plan.topk_idx, plan.D1, plan.chunk_off, plan.rail, plan.S, plan.R, plan.stats)]
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step(True)
        torch.cuda.synchronize()
        for t in (plan.topk_idx, plan.D1, plan.chunk_off, plan.rail, plan.S, plan.R, plan.stats):
            t.zero_()
        for _ in range(max(args.warmup, 1)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        assert all(torch.equal(a, b) for a, b in zip(want_g, (plan.topk_idx, plan.D1, plan.chunk_off, plan.rail, plan.S, plan.R, plan.stats)))
        del graph, want_g

        # ---- supplementary: the plain per-chunk LPT kernel on the same records (same outputs, no closed-form periods)
        rail2, S2 = torch.empty_like(plan.rail), torch.empty_like(plan.S)
        cw = []
        for i in range(3 + min(args.steps, 10)):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            rs.lpt_spray(plan.chunk_off, plan.chunk_w, B, topo, out=(rail2, S2), chunkwise=True)
            e1.record()
            cw.append((e0, e1))
        torch.cuda.synchronize()
        chunkwise_ms = sum(a.elapsed_time(b) for a, b in cw[3:]) / max(len(cw) - 3, 1)
        assert torch.equal(rail2[:total_chunks], plan.rail[:total_chunks]) and torch.equal(S2, plan.S)
        stats = plan.stats.cpu().numpy()
        ratio = stats[:, 0] / np.maximum(stats[:, 3], 1)

        # ---- supplementary: the comparison schemes on the same chunk records, and the second all-to-all (transposed traffic)
        def timed(fn):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fn(); e0.record(); fn(); e1.record(); torch.cuda.synchronize()
            return e0.elapsed_time(e1)
        R2, stats2 = torch.empty_like(plan.R), torch.empty_like(plan.stats)
        schemes = {"lpt": {"makespan_over_lb_max": float(ratio.max()), "makespan_over_lb_mean": float(ratio.mean())}}
        for pol in ("nic_direct", "flow_hash", "random_spray", "round_robin"):
            ms = timed(lambda: rs.assign_policy(pol, 1, plan.chunk_off, plan.chunk_w, plan.chunk_flow, B, topo, out=(rail2, S2)))
            rs.eval(plan.chunk_off, plan.chunk_w, plan.chunk_flow, rail2, S2, B, topo, out=(R2, stats2), ws=plan.ws_eval)
            st2 = stats2.cpu().numpy()
            r2 = st2[:, 0] / np.maximum(st2[:, 3], 1)
            schemes[pol] = {"makespan_over_lb_max": float(r2.max()), "makespan_over_lb_mean": float(r2.mean()), "assign_ms": ms}
        D1T = torch.empty_like(plan.D1)
        tr_ms = timed(lambda: rs.transpose_matrix(plan.D1, topo, out=D1T))
        n_comb = int(rs.chunk_count(D1T, topo, plan.ws_sort)[-1].item())
        plan_c = rs.Plan(topo, B, n_comb, dev, want_perm=True)
        comb_ms = timed(lambda: plan_c.schedule_one_call(D1T))
        st_c = plan_c.stats.cpu().numpy()
        r_c = st_c[:, 0] / np.maximum(st_c[:, 3], 1)
        combine = {"transpose_ms": tr_ms, "schedule_ms": comb_ms, "chunks": n_comb, "makespan_over_lb_max": float(r_c.max())}
        # ---- chunk granularity (Theorem 4): the same traffic matrices cut at other chunk sizes
        sweep = []
        for cb in (16384, 65536, 262144, 1048576, 4194304):
            topo_g = rs.Topo(cfg.M, cfg.N, cb, cfg.rail_bw_Bps)
            n_g = int(rs.chunk_count(plan.D1, topo_g)[-1].item())
            plan_g = rs.Plan(topo_g, B, n_g, dev, want_perm=True)
            ms_g = timed(lambda: plan_g.schedule_one_call(plan.D1))
            st_g, S_g = plan_g.stats.cpu().numpy(), plan_g.S.cpu().numpy().astype(np.float64)
            mse = ((S_g - S_g.mean(axis=2, keepdims=True)) ** 2).mean(axis=2).max(axis=1)      # worst node of each matrix
            wmax = np.maximum(st_g[:, 5], 1).astype(np.float64)
            sweep.append({"chunk_bytes": cb, "chunks": n_g, "schedule_ms": ms_g,
                          "makespan_over_lb_max": float((st_g[:, 0] / np.maximum(st_g[:, 3], 1)).max()),
                          "send_spread_over_wmax_max": float((st_g[:, 7] / wmax).max()),
                          "mse_over_wmax2_max": float((mse / (wmax * wmax)).max())})
            del plan_g
        # ---- expert placement (Section 6.3, sparse against dense): the first R replica groups of the placement table only
        placement = []
        for R_ in sorted({1, 2, max(cfg.replicas // 2, 1), cfg.replicas}):
            eg_R = torch.from_numpy(np.ascontiguousarray(eg_np[:, :R_])).to(dev)
            _, D1_R = rs.route_traffic(logits, cfg.k, B, cfg.tokens_per_gpu, eg_R, cfg.payload_bytes, topo, out=(plan.topk_idx, D1T), ws=ws_rt)
            n_R = int(rs.chunk_count(D1_R, topo)[-1].item())
            plan_R = rs.Plan(topo, B, n_R, dev, want_perm=True)
            ms_R = timed(lambda: plan_R.schedule_one_call(D1_R))
            st_R = plan_R.stats.cpu().numpy()
            placement.append({"replicas": R_, "gpus_with_experts": R_ * (cfg.E // cfg.experts_per_gpu), "chunks": n_R, "schedule_ms": ms_R,
                              "makespan_over_lb_max": float((st_R[:, 0] / np.maximum(st_R[:, 3], 1)).max()),
                              "completion_time_us_max": float(st_R[:, 0].max() / cfg.rail_bw_Bps * 1e6)})
            del plan_R
        rs.chunk_sort(plan.D1, topo, capacity=plan.capacity, out=(plan.chunk_off, plan.chunk_w, plan.chunk_flow, plan.perm), ws=plan.ws_sort)

    # ---- roofline of the dominant kernel (route_traffic streams the logits once and writes the indices once)
    k1_bytes = rows * (4 * cfg.E + 4 * cfg.k)
    k2_bytes = rows * 4 * cfg.k + 8 * B * G * G
    rt_bytes = k1_bytes + 8 * B * G * G
    rt_gbps = rt_bytes / (stage_ms["route_traffic"] * 1e-3) / 1e9
    k1_gbps = k1_bytes / (staged_ms["route_topk"] * 1e-3) / 1e9
    staged_routing_gbps = (k1_bytes + k2_bytes) / ((staged_ms["route_topk"] + staged_ms["traffic_matrix"]) * 1e-3) / 1e9
    dominant = max(stage_ms, key=stage_ms.get)
    # the per-chunk LPT kernel against the VALU issue rate: ceil(log2 N) cross-lane mins + add, compare, select and the
    # shift that files the decision, per greedy step and wavefront (one instance per wavefront at this instance count);
    # 256 CUs x 4 SIMDs issue one wave64 VALU instruction per 4 cycles at 2.4 GHz
    gw = 4 if cfg.N <= 4 else 8 if cfg.N <= 8 else 16 if cfg.N <= 16 else 32 if cfg.N <= 32 else 64
    ipw = 64 // gw if B * cfg.M >= 2048 * 64 // gw else 1
    instr_per_step = gw.bit_length() - 1 + 5
    valu_peak = 256 * 4 * 2.4e9 / 4 / 1e9            # G wave-instructions/s
    lpt_rate = total_chunks / (staged_ms["lpt_spray"] * 1e-3)

    out = {
        "metric": "LPT-sprayed chunks/s over the whole path (route_topk, traffic_matrix, chunk_sort, lpt_spray, eval; stages 1-2 and 3-5 fused into two calls)",
        "value": total_chunks / (ms_per_step * 1e-3),
        "unit": "chunks/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64 loads / uint32 weights / fp32 compare-only",
        "data": "synthetic (seeded counter-based logits, Zipf expert bias)",
        "config": {"workload": f"{cfg.name}: Mixtral-8x7B-shaped, M={cfg.M} nodes x N={cfg.N} rails, E={cfg.E} top-{cfg.k}, "
                               f"{cfg.tokens_per_gpu} tokens/GPU x {cfg.payload_bytes} B, C={cfg.chunk_bytes} B, {B} matrices of {G}x{G}",
                   "rows": rows, "chunks": total_chunks, "instances": B * cfg.M},
        "stage_ms": stage_ms,
        "staged": {"ms_per_step": staged_ms_per_step, "value": total_chunks / (staged_ms_per_step * 1e-3), "stage_ms": staged_ms,
                   "note": "the same step through the five separate calls (indices written, then read back)",
                   "route_topk_GBps": k1_gbps, "routing_to_traffic_matrix_GBps": staged_routing_gbps},
        "two_steps_in_flight": None if piped_ms is None else {
            "ms_per_step": piped_ms, "value": total_chunks / (piped_ms * 1e-3),
            "note": "same two calls per step, consecutive steps alternating between two streams and two sets of outputs"},
        "graph_replay": None if graph_ms is None else {
            "ms_per_step": graph_ms, "value": total_chunks / (graph_ms * 1e-3),
            "note": "the same two calls captured once into a HIP graph and replayed; outputs checked against the eager step"},
        "routing_to_traffic_matrix_GBps": rt_gbps,
        "routing_frac_of_hbm_peak": rt_gbps / HBM_PEAK_GBPS,
        "lpt_spray_chunks_per_s": lpt_rate,
        "lpt_roofline": None if chunkwise_ms is None else {
            "kernel": "railsched_lpt_spray_chunkwise", "bound": "alu", "unit": "G wave-instr/s", "peak": valu_peak,
            "achieved": total_chunks / ipw * instr_per_step / (chunkwise_ms * 1e-3) / 1e9,
            "frac": total_chunks / ipw * instr_per_step / (chunkwise_ms * 1e-3) / 1e9 / valu_peak,
            "note": f"{B * cfg.M} instances are {B * cfg.M // ipw} wavefronts on 1024 SIMDs: the latency of the serial chain "
                    f"({instr_per_step} instructions per step), not the issue rate, bounds this workload"},
        "lpt_spray_chunkwise_ms": chunkwise_ms,
        "makespan_over_lower_bound": {"max": float(ratio.max()), "mean": float(ratio.mean())},
        "schemes": schemes,
        "granularity_sweep": sweep,
        "placement_sweep": placement,
        "second_all_to_all": combine,
        "completion_time_us_max": float(stats[:, 0].max() / cfg.rail_bw_Bps * 1e6),
        "roofline": {"kernel": "route_traffic_kernel (with rt_reduce_kernel, the sum of its slice counts, in the same call)",
                     "bound": "hbm", "achieved": rt_gbps, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": rt_gbps / HBM_PEAK_GBPS,
                     "traffic": ROUTE_TRAFFIC_C2_TRAFFIC_BYTES if cfg.name == "c2" else None,
                     "algorithmic_bytes_per_launch": rt_bytes, "avg_launch_ms": stage_ms["route_traffic"],
                     "slowest_stage": dominant},
    }

    # ---- CPU baseline: the oracle as it stands, on the first layers of the same workload
    if args.cpu_layers != 0:
        import oracle
        L = B if args.cpu_layers < 0 else min(args.cpu_layers, B)
        x = logits[: L * cfg.rows_per_layer].cpu().numpy()

        def cpu_path(xs, layers):
            idx = oracle.route_topk(xs, cfg.k)
            D1c = oracle.traffic_matrix(idx, layers, cfg.tokens_per_gpu, eg_np, cfg.payload_bytes, cfg.M, cfg.N)
            off, w, flow, _ = oracle.chunk_sort_batch(D1c, cfg.M, cfg.N, cfg.chunk_bytes)
            rail, S = oracle.lpt_batch(off, w, layers, cfg.M, cfg.N)
            _, R, stats = oracle.eval_batch(off, w, flow, rail, layers, cfg.M, cfg.N)
            return off, rail, R, stats
        c0 = time.perf_counter()
        off_c, rail_c, R_c, stats_c = cpu_path(x, L)
        c1 = time.perf_counter()
        n_c = int(off_c[-1])
        # the same oracle on one thread, on the first quarter of the sample
        L1 = max(L // 4, 1)
        all_threads = oracle.num_threads()
        oracle.set_threads(1)
        s0 = time.perf_counter()
        off_1 = cpu_path(x[: L1 * cfg.rows_per_layer], L1)[0]
        s1 = time.perf_counter()
        oracle.set_threads(all_threads)
        same = (np.array_equal(plan.stats[:L].cpu().numpy(), stats_c)
                and np.array_equal(plan.rail[:n_c].cpu().numpy(), rail_c)
                and np.array_equal(plan.R[:L].cpu().numpy(), R_c))
        out["cpu_baseline"] = {"value": n_c / (c1 - c0), "unit": "chunks/s", "cores": all_threads, "kind": "oracle",
                               "sample": f"first {L} of {B} layers ({L * cfg.rows_per_layer} rows, {n_c} chunks), whole path, "
                                         f"{c1 - c0:.2f} s", "matches_gpu": bool(same),
                               "single_thread": {"value": int(off_1[-1]) / (s1 - s0), "unit": "chunks/s", "cores": 1,
                                                 "sample": f"first {L1} layers, {s1 - s0:.2f} s"}}
    print(json.dumps(out))


def _events(torch):
    e = torch.cuda.Event(enable_timing=True)
    e.record()
    return e


def _stage_rooflines(total_chunks, n_inst, topo, ms, want_perm):
    """GB/s of stages 3-5 on their algorithmic bytes: D1 read + 8 (12 with perm) B per chunk; 4 + 1 B; 9 B."""
    NG = topo.rails * topo.G
    by = {"chunk_sort": 8 * NG * n_inst + (12 if want_perm else 8) * total_chunks,
          "lpt_spray": 5 * total_chunks, "eval": 9 * total_chunks}
    return {n: {"GBps": by[n] / (ms[n] * 1e-3) / 1e9, "frac_of_hbm_peak": by[n] / (ms[n] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                "algorithmic_bytes": by[n]} for n in by}


def _schedule_steps(rs, torch, plan, D1, topo, B, steps, warmup):
    """Per-stage times of stages 3-5 through the three calls, and the time of railsched_schedule on the same input."""
    names = ("chunk_sort", "lpt_spray", "eval")
    ms = {n: 0.0 for n in names}
    for it in range(warmup + steps):
        e = [_events(torch)]
        rs.chunk_sort(D1, topo, capacity=plan.capacity, out=(plan.chunk_off, plan.chunk_w, plan.chunk_flow, plan.perm), ws=plan.ws_sort)
        e.append(_events(torch))
        rs.lpt_spray(plan.chunk_off, plan.chunk_w, B, topo, out=(plan.rail, plan.S))
        e.append(_events(torch))
        rs.eval(plan.chunk_off, plan.chunk_w, plan.chunk_flow, plan.rail, plan.S, B, topo, out=(plan.R, plan.stats), ws=plan.ws_eval)
        e.append(_events(torch))
        torch.cuda.synchronize()
        if it >= warmup:
            for i, n in enumerate(names):
                ms[n] += e[i].elapsed_time(e[i + 1]) / steps
    small = [t.clone() for t in (plan.chunk_off, plan.S, plan.R, plan.stats)]
    rail3 = plan.rail.clone()
    for t in (plan.rail, plan.S, plan.R, plan.stats):
        t.zero_()
    one = 0.0
    for it in range(warmup + steps):
        e0 = _events(torch)
        plan.schedule_one_call(D1)
        e1 = _events(torch)
        torch.cuda.synchronize()
        if it >= warmup:
            one += e0.elapsed_time(e1) / steps
    assert all(torch.equal(a, b) for a, b in zip(small, (plan.chunk_off, plan.S, plan.R, plan.stats))) and torch.equal(rail3, plan.rail)
    return ms, one


def bench_flows(cfg, args, rs, W, torch, np):
    """c3 / c5: no routing stage; a step is stages 3-5 over `--matrices` synthetic flow matrices resident in HBM."""
    dev = "cuda:0"
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes, cfg.rail_bw_Bps)
    B = args.matrices if args.matrices > 0 else (cfg.batch if cfg.G <= 256 else 1)
    want_perm = cfg.G <= 256                       # the permutation of a 3.9e9-chunk matrix is left out (16 GB more)
    D1 = W.gen_flow_matrices_device(cfg, dev, first=0, count=B)
    total = int(rs.chunk_count(D1, topo)[-1].item())
    plan = rs.Plan(topo, B, total, dev, want_perm=want_perm)
    steps, warmup = min(args.steps, 5), min(args.warmup, 2)
    ms, one_ms = _schedule_steps(rs, torch, plan, D1, topo, B, steps, warmup)
    step_ms = one_ms
    st = plan.stats.cpu().numpy()
    ratio = st[:, 0] / np.maximum(st[:, 3], 1)
    per_chunk = None
    if not args.skip_extras:
        # the per-chunk kernel (every chunk through the cross-lane argmin) on the same records, against the VALU issue rate
        rail2, S2 = torch.empty_like(plan.rail), torch.empty_like(plan.S)
        t = []
        for _ in range(3):
            e0, e1 = _events(torch), None
            rs.lpt_spray(plan.chunk_off, plan.chunk_w, B, topo, out=(rail2, S2), chunkwise=True)
            e1 = _events(torch)
            torch.cuda.synchronize()
            t.append(e0.elapsed_time(e1))
        assert torch.equal(rail2, plan.rail) and torch.equal(S2, plan.S)
        del rail2, S2
        gw = 4 if cfg.N <= 4 else 8 if cfg.N <= 8 else 16 if cfg.N <= 16 else 32 if cfg.N <= 32 else 64
        ipw = 64 // gw if B * cfg.M >= 2048 * 64 // gw else 1                      # instances per wavefront (packed or wide shape)
        instr = (gw.bit_length() - 1) + (4 if ipw > 1 else 5)                     # cross-lane mins + add, compare, select, decision filed (+ weight broadcast)
        valu_peak = 256 * 4 * 2.4e9 / 4
        per_chunk = {"ms": min(t[1:]), "chunks_per_s": total / (min(t[1:]) * 1e-3), "instances_per_wavefront": ipw,
                     "roofline": {"bound": "alu", "unit": "G wave-instr/s", "peak": valu_peak / 1e9,
                                  "achieved": total / ipw * instr / (min(t[1:]) * 1e-3) / 1e9,
                                  "frac": total / ipw * instr / (min(t[1:]) * 1e-3) / valu_peak,
                                  "note": f"{instr} VALU instructions per greedy step and wavefront, {ipw} instance(s) per wavefront; "
                                          "256 CUs x 4 SIMDs x 2.4 GHz / 4 clocks per wave64 instruction"}}
    roof = _stage_rooflines(total, B * cfg.M, topo, ms, want_perm)
    one_bytes = 8 * topo.rails * topo.G * B * cfg.M + (13 if want_perm else 9) * total
    slow = max(ms, key=ms.get)
    print(json.dumps({
        "metric": "LPT-sprayed chunks/s over stages 3-5 (chunk_sort, lpt_spray, eval, in one call); the workload has no routing stage",
        "value": total / (step_ms * 1e-3), "unit": "chunks/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64 loads / uint32 weights", "data": "synthetic (seeded lognormal flow matrices)",
        "config": {"workload": f"{cfg.name}: M={cfg.M} nodes x N={cfg.N} rails, {B} of {cfg.batch} matrices of {cfg.G}x{cfg.G}, "
                               f"C={cfg.chunk_bytes} B, p_zero={cfg.p_zero}", "chunks": total, "instances": B * cfg.M, "perm": want_perm},
        "timing": "event time of railsched_schedule (stages 3-5 in one call); the three separate calls under `staged`",
        "stage_ms": {"schedule": one_ms},
        "staged": {"ms_per_step": sum(ms.values()), "stage_ms": ms, "stage_rooflines": roof},
        "lpt_spray_chunks_per_s": total / (ms["lpt_spray"] * 1e-3),
        "lpt_spray_per_chunk_kernel": per_chunk,
        "makespan_over_lower_bound": {"max": float(ratio.max()), "mean": float(ratio.mean())},
        "roofline": {"kernel": "railsched_schedule (cs_fill_kernel dominates: records and leading-run rails written once)",
                     "bound": "hbm", "achieved": one_bytes / (one_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": one_bytes / (one_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, "traffic": None,
                     "algorithmic_bytes_per_launch": one_bytes},
    }))


def bench_streamed(cfg, args, rs, W, torch, np):
    """c4: the logits of all layers do not fit beside the records, so each layer's logits are generated into one
    buffer (untimed), stages 1-2 are timed per layer, and stages 3-5 run once over all matrices."""
    dev = "cuda:0"
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes, cfg.rail_bw_Bps)
    B, G = cfg.batch, cfg.G
    expert_gpu = torch.from_numpy(W.expert_gpu_table(cfg)).to(dev)
    D1 = torch.empty((B, G, G), dtype=torch.int64, device=dev)
    idx = torch.empty((cfg.rows_per_layer, cfg.k), dtype=torch.int32, device=dev)
    t1 = t2 = 0.0
    for b in range(B):
        lg = W.gen_logits(cfg, b, device=dev)
        if b == 0:
            rs.route_topk(lg, cfg.k, out=idx)           # warm-up launch
        e0 = _events(torch)
        rs.route_topk(lg, cfg.k, out=idx)
        e1 = _events(torch)
        rs.traffic_matrix(idx, 1, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo, out=D1[b:b + 1])
        e2 = _events(torch)
        torch.cuda.synchronize()
        t1 += e0.elapsed_time(e1)
        t2 += e1.elapsed_time(e2)
        del lg
    del idx
    total = int(rs.chunk_count(D1, topo)[-1].item())
    plan = rs.Plan(topo, B, total, dev, want_perm=True)
    steps, warmup = min(args.steps, 5), min(args.warmup, 2)
    ms3, one_ms = _schedule_steps(rs, torch, plan, D1, topo, B, steps, warmup)
    ms = {"route_topk": t1, "traffic_matrix": t2, "schedule": one_ms}
    step_ms = sum(ms.values())
    rows = B * cfg.rows_per_layer
    k1_bytes = rows * (4 * cfg.E + 4 * cfg.k)
    k2_bytes = rows * 4 * cfg.k + 8 * B * G * G
    st = plan.stats.cpu().numpy()
    ratio = st[:, 0] / np.maximum(st[:, 3], 1)
    k1_gbps = k1_bytes / (t1 * 1e-3) / 1e9
    print(json.dumps({
        "metric": "LPT-sprayed chunks/s over the whole path (route_topk, traffic_matrix, chunk_sort, lpt_spray, eval)",
        "value": total / (step_ms * 1e-3), "unit": "chunks/s", "n_gpus": 1, "steps": 1, "warmup": 1,
        "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64 loads / uint32 weights / fp32 compare-only", "data": "synthetic (seeded counter-based logits, Zipf expert bias)",
        "config": {"workload": f"{cfg.name}: M={cfg.M} nodes x N={cfg.N} rails, E={cfg.E} top-{cfg.k}, {cfg.tokens_per_gpu} tokens/GPU x "
                               f"{cfg.payload_bytes} B, C={cfg.chunk_bytes} B, {B} matrices of {G}x{G}", "rows": rows, "chunks": total,
                   "instances": B * cfg.M},
        "timing": "sum of event times: stages 1-2 once per layer (logits regenerated between layers, untimed), stages 3-5 (one call) averaged over steps",
        "stage_ms": ms, "staged": {"stage_ms": ms3, "stage_rooflines": _stage_rooflines(total, B * cfg.M, topo, ms3, True)},
        "routing_to_traffic_matrix_GBps": (k1_bytes + k2_bytes) / ((t1 + t2) * 1e-3) / 1e9,
        "makespan_over_lower_bound": {"max": float(ratio.max()), "mean": float(ratio.mean())},
        "roofline": {"kernel": "route_topk_merge_kernel", "bound": "hbm", "achieved": k1_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": k1_gbps / HBM_PEAK_GBPS, "traffic": None, "algorithmic_bytes_per_launch": k1_bytes // B,
                     "avg_launch_ms": t1 / B,
                     "note": "for E = 256, k = 8 the kernel issues 925 VALU instructions per wavefront of 8 rows: "
                             "rows/8 x 925 x 4 clocks / (1024 SIMDs x 2.4 GHz) is within a few percent of the launch time, "
                             "so it is bound by VALU issue as much as by HBM"},
    }))


if __name__ == "__main__":
    main()
