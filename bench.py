#!/usr/bin/env python3
"""Benchmark of the whole rail-spraying path on one MI355X.

A step is one pass of all five stages (route_topk -> traffic_matrix -> chunk_sort -> lpt_spray ->
eval) over one batch of the Mixtral-8x7B-shaped workload: 8 nodes x 8 rails, 8 experts top-2,
16384 tokens per GPU, 8 KiB tokens, 256 KiB chunks, 32 layers = 32 traffic matrices of 64x64.
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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c2", help="workload (c1, c2; default c2 = the benchmark workload)")
    ap.add_argument("--cpu-layers", type=int, default=8, help="layers of the workload the CPU oracle is timed on (0 = skip)")
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
    assert cfg.kind == "moe"
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes, cfg.rail_bw_Bps)
    B, G = cfg.batch, cfg.G
    rows = B * cfg.rows_per_layer

    # ---- inputs, resident in HBM
    logits = torch.empty((rows, cfg.E), dtype=torch.float32, device=dev)
    for b in range(B):
        logits[b * cfg.rows_per_layer:(b + 1) * cfg.rows_per_layer] = W.gen_logits(cfg, b, device=dev)
    eg_np = W.expert_gpu_table(cfg)
    expert_gpu = torch.from_numpy(eg_np).to(dev)

    # ---- size the record arrays once (count query), then a plan that allocates nothing per step
    idx0 = rs.route_topk(logits, cfg.k)
    D10 = rs.traffic_matrix(idx0, B, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo)
    total_chunks = int(rs.chunk_count(D10, topo)[-1].item())
    del idx0, D10
    plan = rs.Plan(topo, B, total_chunks, dev, rows=rows, k=cfg.k, want_perm=True)

    names = ("route_topk", "traffic_matrix", "chunk_sort", "lpt_spray", "eval")

    def step(events=None):
        marks = []
        def mark():
            if events is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                marks.append(e)
        mark()
        rs.route_topk(logits, cfg.k, out=plan.topk_idx); mark()
        rs.traffic_matrix(plan.topk_idx, B, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo, out=plan.D1); mark()
        rs.chunk_sort(plan.D1, topo, capacity=plan.capacity,
                      out=(plan.chunk_off, plan.chunk_w, plan.chunk_flow, plan.perm), ws=plan.ws_sort); mark()
        rs.lpt_spray(plan.chunk_off, plan.chunk_w, B, topo, out=(plan.rail, plan.S)); mark()
        rs.eval(plan.chunk_off, plan.chunk_w, plan.chunk_flow, plan.rail, plan.S, B, topo,
                out=(plan.R, plan.stats), ws=plan.ws_eval); mark()
        if events is not None:
            events.append(marks)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(ev)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    stage_ms = {n: 0.0 for n in names}
    for marks in ev:
        for i, n in enumerate(names):
            stage_ms[n] += marks[i].elapsed_time(marks[i + 1])
    stage_ms = {n: v / args.steps for n, v in stage_ms.items()}

    assert int(plan.chunk_off[-1].item()) == total_chunks
    stats = plan.stats.cpu().numpy()
    ratio = stats[:, 0] / np.maximum(stats[:, 3], 1)

    # ---- roofline of the dominant kernel (route_topk streams the logits once)
    k1_bytes = rows * (4 * cfg.E + 4 * cfg.k)
    k2_bytes = rows * 4 * cfg.k + 8 * B * G * G
    k1_gbps = k1_bytes / (stage_ms["route_topk"] * 1e-3) / 1e9
    routing_gbps = (k1_bytes + k2_bytes) / ((stage_ms["route_topk"] + stage_ms["traffic_matrix"]) * 1e-3) / 1e9
    dominant = max(stage_ms, key=stage_ms.get)

    out = {
        "metric": "LPT-sprayed chunks/s over the whole path (route_topk, traffic_matrix, chunk_sort, lpt_spray, eval)",
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
        "routing_to_traffic_matrix_GBps": routing_gbps,
        "routing_frac_of_hbm_peak": routing_gbps / HBM_PEAK_GBPS,
        "lpt_spray_chunks_per_s": total_chunks / (stage_ms["lpt_spray"] * 1e-3),
        "makespan_over_lower_bound": {"max": float(ratio.max()), "mean": float(ratio.mean())},
        "completion_time_us_max": float(stats[:, 0].max() / cfg.rail_bw_Bps * 1e6),
        "roofline": {"kernel": "route_topk_kernel", "bound": "hbm", "achieved": k1_gbps, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": k1_gbps / HBM_PEAK_GBPS, "traffic": None,
                     "algorithmic_bytes_per_launch": k1_bytes, "avg_launch_ms": stage_ms["route_topk"],
                     "slowest_stage": dominant},
    }

    # ---- CPU baseline: the oracle as it stands, on the first layers of the same workload
    if args.cpu_layers > 0:
        import oracle
        L = min(args.cpu_layers, B)
        x = logits[: L * cfg.rows_per_layer].cpu().numpy()
        c0 = time.perf_counter()
        idx_c = oracle.route_topk(x, cfg.k)
        D1_c = oracle.traffic_matrix(idx_c, L, cfg.tokens_per_gpu, eg_np, cfg.payload_bytes, cfg.M, cfg.N)
        off_c, w_c, flow_c, perm_c = oracle.chunk_sort_batch(D1_c, cfg.M, cfg.N, cfg.chunk_bytes)
        rail_c, S_c = oracle.lpt_batch(off_c, w_c, L, cfg.M, cfg.N)
        _, R_c, stats_c = oracle.eval_batch(off_c, w_c, flow_c, rail_c, L, cfg.M, cfg.N)
        c1 = time.perf_counter()
        n_c = int(off_c[-1])
        same = (np.array_equal(plan.stats[:L].cpu().numpy(), stats_c)
                and np.array_equal(plan.rail[:n_c].cpu().numpy(), rail_c)
                and np.array_equal(plan.R[:L].cpu().numpy(), R_c))
        out["cpu_baseline"] = {"value": n_c / (c1 - c0), "unit": "chunks/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"first {L} of {B} layers ({L * cfg.rows_per_layer} rows, {n_c} chunks), whole path, "
                                         f"{c1 - c0:.2f} s", "matches_gpu": bool(same)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
