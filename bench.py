#!/usr/bin/env python3
"""Benchmark of the rail-spraying path on one MI355X.  Prints ONE JSON line.

Headline (metric, value, ms_per_step): the Mixtral-8x7B-shaped workload c2 - 8 nodes x 8 rails, 8 experts
top-2, 16384 tokens per GPU, 8 KiB tokens, 256 KiB chunks, 32 layers = 32 traffic matrices of 64x64 - with its
1 GiB of fp32 router logits resident in HBM before timing starts.  A step is one pass of all five stages
(route_topk -> traffic_matrix -> chunk_sort -> lpt_spray -> eval) through two calls: railsched_route_traffic
(stages 1-2 in one pass over the logits) and railsched_schedule (stages 3-5).  Both write the same bytes as
the five separate calls - asserted here on every output array; the five calls are timed too ("staged").

Beside it, under "workloads", one record for each larger workload, each with the rooflines of its calls, the
per-chunk LPT kernel against the VALU issue rate, and the CPU oracle timed in the same run on a stated sample:
  c3  sparse synthetic flows, 32 x 8, 1024 matrices of 256x256 resident (3.9e9 chunks, 32 768 instances): stages 3-5
  c4  DeepSeek-V3-shaped, 64 x 8, 256 experts top-8, 61 layers of 4 194 304 rows: whole path, one layer's 4 GiB of
      logits resident at a time (regenerated between layers, untimed)
  c5  stress, 128 x 8, all 256 matrices of 1024x1024, one matrix (3.9e9 chunks) resident at a time: stages 3-5
--config c1|c2|c3|c4|c5 runs that workload alone (its record is the whole line); used for the profiles.
Stage times are medians over the repetitions (hipEvents on the stream the calls are enqueued on).
"""
import argparse
import hashlib
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0                      # MI355X published HBM3E bandwidth
VALU_PEAK_GIPS = 256 * 4 * 2.4e9 / 4 / 1e9  # G wave-instructions/s: 256 CUs x 4 SIMDs, one wave64 VALU instruction per 4 clocks at 2.4 GHz


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="all",
                    help="all (default): c2 as the headline and c3, c4, c5 as sub-records; c1..c5: that workload alone")
    ap.add_argument("--matrices", type=int, default=0, help="c3/c5: matrices to run (0 = all)")
    ap.add_argument("--layers", type=int, default=0, help="c4: layers to run (0 = all 61)")
    ap.add_argument("--cpu-layers", type=int, default=-1,
                    help="c1/c2: layers the CPU oracle is timed on (-1 = all, 0 = skip every CPU baseline)")
    ap.add_argument("--skip-extras", action="store_true",
                    help="only the timed regions: no supplementary measurements (used for profiles, so that a kernel's "
                         "average duration is that of the timed region)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device copy first: a kernel of known traffic to scale profiler byte counters by")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------------ helpers
def _event(torch):
    e = torch.cuda.Event(enable_timing=True)
    e.record()
    return e


def _median(xs):
    return float(statistics.median(xs)) if xs else None


def _sha12(source):
    """First 12 hex digits of the sha256 of a kernel source file followed by every header of the library (sorted by name)."""
    csrc = os.path.join(ROOT, "paper_2510_19262_amd", "csrc")
    h = hashlib.sha256()
    for name in [source] + sorted(f for f in os.listdir(csrc) if f.endswith(".h")):
        with open(os.path.join(csrc, name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:12]


def counter_traffic(kernels, workload):
    """HBM bytes per launch of `kernels` (one name, or several whose launches make up one call) on `workload`, from the
    rocprofv3 counter runs summarised under profiles/ (FETCH_SIZE and WRITE_SIZE, each scaled by what it reads for a copy
    of known size).  The summaries carry lines
      TRAFFIC <kernel> <workload> read_MiB=<x> written_MiB=<y> source=<file under csrc> sha=<see _sha12>
    and this is the one place the benchmark takes the figure from.  None when a kernel has no such line, or when its
    source (or a header of the library) has changed since the counters were taken."""
    pdir = os.path.join(ROOT, "profiles")
    if not os.path.isdir(pdir):
        return None
    pat = re.compile(r"^TRAFFIC\s+(\S+)\s+(\S+)\s+read_MiB=([0-9.]+)\s+written_MiB=([0-9.]+)\s+source=(\S+)\s+sha=([0-9a-f]+)")
    found = {}
    for name in sorted(os.listdir(pdir)):
        if not name.endswith((".md", ".txt")):
            continue
        for line in open(os.path.join(pdir, name)):
            m = pat.match(line.strip())
            if m and m.group(2) == workload and m.group(1) not in found:
                found[m.group(1)] = m
    total = 0.0
    for k in ([kernels] if isinstance(kernels, str) else kernels):
        m = found.get(k) or found.get(k.split(":")[0])   # "<kernel>:one_call" lines exist only where that dispatch differs
        if m is None or not os.path.exists(os.path.join(ROOT, "paper_2510_19262_amd", "csrc", m.group(5))) or _sha12(m.group(5)) != m.group(6):
            return None
        total += float(m.group(3)) + float(m.group(4))
    return int(total * 1024 * 1024)


def copy_probe(torch, dev):
    """One 1 GiB device-to-device copy: a kernel whose traffic is known, to scale the profiler's byte counters by."""
    src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


MEASURED = {}


def measure_streams(torch, dev, reps=7):
    """What this machine's HBM sustains for a plain copy (1 GiB read + 1 GiB written) and a plain fill (1 GiB written), timed like
    the stages: the rooflines quote their rate against the published peak and, as `frac_of_measured_copy`, against the first."""
    src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    res = {}
    for name, fn, nbytes in (("copy", lambda: dst.copy_(src), 2 << 30), ("fill", lambda: dst.fill_(1.0), 1 << 30)):
        ts = []
        for _ in range(reps):
            e0 = _event(torch)
            fn()
            e1 = _event(torch)
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        res[name + "_GBps"] = nbytes / (_median(ts[1:]) * 1e-3) / 1e9
    del src, dst
    MEASURED.update(res)
    return res


def profiled_kernel_us(kernel, workload):
    """Average duration (us) of `kernel` in the rocprofv3 --kernel-trace --stats run summarised under profiles/ for `workload`
    (first table of the summary; the average runs over every call of the kernel in that run), or None."""
    pdir = os.path.join(ROOT, "profiles")
    if not os.path.isdir(pdir):
        return None
    for name in sorted(os.listdir(pdir)):
        if not name.startswith(workload + "_") or not name.endswith((".md", ".txt")):
            continue
        in_table = False
        for line in open(os.path.join(pdir, name)):
            if line.startswith("## "):
                in_table = line.startswith("## Kernel durations")
            elif in_table and line.startswith("| " + kernel):
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                try:
                    return float(cells[2])
                except (IndexError, ValueError):
                    return None
    return None


def write_probe(torch, plan, total, reps=5):
    """Plain fills of the record arrays a schedule call writes (weights, flows, the permutation if kept, rails), `total`
    records each: the same bytes written by a kernel that does nothing else (torch's fill, one launch per array; the rail
    bytes are filled as 32-bit words like the others), timed in the same run as the record fill.  The arrays are scratch
    outputs that the next call rewrites."""
    # lengths cut to multiples of 2^20 words: torch splits a tensor of more than 2^31 elements into halves, and halves of an odd
    # length start off the 16-byte grid, which sends its fill down an unvectorised path (4.8 instead of 6.8 TB/s)
    cut = lambda n: n - n % (1 << 20)
    arrs = [a[:cut(total)] for a in (plan.chunk_w, plan.chunk_flow, plan.perm) if a is not None]
    arrs.append(plan.rail[:4 * cut(total // 4)].view(torch.int32))
    arrs = [a for a in arrs if a.numel()]
    nbytes = sum(a.numel() * a.element_size() for a in arrs)
    if nbytes == 0:
        return None
    ts = []
    for _ in range(reps):
        e0 = _event(torch)
        for a in arrs:
            a.fill_(1)
        e1 = _event(torch)
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    ms = _median(ts)
    return {"what": "torch fill_ of the record arrays of one schedule call (%d arrays, one launch each)" % len(arrs),
            "bytes": nbytes, "ms": ms, "GB/s": nbytes / (ms * 1e-3) / 1e9, "frac_of_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}


def hbm_roofline(kernel, workload, algorithmic_bytes, ms, note=None, counted=None):
    """`counted`: the kernels whose counter traffic adds up to the call (default: the kernel named first in `kernel`)."""
    gbps = algorithmic_bytes / (ms * 1e-3) / 1e9
    r = {"kernel": kernel, "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
         "traffic": counter_traffic(counted or COUNTED.get(kernel, kernel.split(" ")[0]), workload),
         "algorithmic_bytes_per_launch": int(algorithmic_bytes),
         "avg_launch_ms": ms}
    if MEASURED.get("copy_GBps"):
        r["frac_of_measured_copy"] = gbps / MEASURED["copy_GBps"]
    us = profiled_kernel_us(kernel.split(" ")[0], workload)
    if us:   # the dominant kernel alone, as the committed profile timed it (the call above also holds its small companions)
        r["profiled_kernel_avg_us"] = us
        r["frac_at_profiled_kernel_time"] = algorithmic_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS
    if note:
        r["note"] = note
    return r


def lpt_alu_roofline(total_chunks, n_inst, N, ms):
    """The per-chunk LPT kernel against the VALU issue rate, in instructions the greedy step needs per wavefront.  The
    library picks the shape by the number of instances (mirrored here):
    wide (one instance per wavefront, loads kept as a sorted list across lanes): 6 instructions per step (weight out of
      its lane, into a vector register, subtract from the head through DPP, neighbour through DPP, median of three, file
      the decision), 7 for N > 16 (the head through v_readfirstlane);
    rows (N <= 16, four instances per wavefront, one sorted list per row of 16 lanes): 5 per step for the four;
    packed (64/GW instances per wavefront, loads by rail): ceil(log2 GW) cross-lane mins, the add, compare, select and the
      instruction that files the decision, for the 64/GW."""
    gw = 4 if N <= 4 else 8 if N <= 8 else 16 if N <= 16 else 32 if N <= 32 else 64
    if gw <= 16:
        shape = "wide" if n_inst <= 1024 else "rows" if (gw == 16 or n_inst <= 16384) else "packed"
    else:
        shape = "packed" if (gw == 32 and n_inst > 5 * 1024) else "wide"
    ipw = {"wide": 1, "rows": 4, "packed": 64 // gw}[shape]
    instr = {"wide": 6 if N <= 16 else 7, "rows": 5, "packed": (gw.bit_length() - 1) + 4}[shape]
    ach = total_chunks / ipw * instr / (ms * 1e-3) / 1e9
    return {"kernel": {"wide": "lpt_wide_kernel<GW,false>", "rows": "lpt_rows_kernel<GW,false,...>", "packed": "lpt_packed_kernel<GW,false,...>"}[shape],
            "bound": "alu", "unit": "G wave-instr/s",
            "peak": VALU_PEAK_GIPS, "achieved": ach, "frac": ach / VALU_PEAK_GIPS, "avg_launch_ms": ms,
            "instructions_per_step": instr, "instances_per_wavefront": ipw, "wavefronts": -(-n_inst // ipw),
            "note": "algorithmic VALU instructions of the greedy step; with fewer wavefronts than 4 per SIMD (1024 SIMDs) the "
                    "latency of the chain, not the issue rate, bounds the kernel"}


def stage_bytes(total_chunks, n_inst, topo, want_perm):
    """Algorithmic HBM bytes of stages 3-5: D1 read + 8 (12 with perm) B written per chunk; 4 B read + 1 B written; 9 B read."""
    NG = topo.rails * topo.G
    return {"chunk_sort": 8 * NG * n_inst + (12 if want_perm else 8) * total_chunks, "lpt_spray": 5 * total_chunks,
            "eval": 9 * total_chunks, "schedule": 8 * NG * n_inst + (13 if want_perm else 9) * total_chunks}


STAGE_KERNEL = {"chunk_sort": "cs_fill_kernel (with the count, scan and tail-sort kernels of the call)",
                "lpt_spray": "lpt_prefix_kernel (with the serial kernel behind the leading runs)",
                "eval": "eval_partial_kernel (with the reduction of the call)",
                "schedule": "cs_fill_kernel (railsched_schedule: records and leading-run rails written once; count, scan, tail sort, "
                            "serial LPT behind the leading runs, closed-form receive loads and reduction in the same call)"}


# the record fill launched by railsched_schedule also writes the leading-run rails: its own counter line
COUNTED = {STAGE_KERNEL["schedule"]: "cs_fill_kernel:one_call"}


def time_stages_3_5(rs, torch, plan, D1, topo, B, reps, warmup):
    """Medians of the three separate calls and of railsched_schedule on the same input; asserts identical outputs."""
    names = ("chunk_sort", "lpt_spray", "eval")
    t = {n: [] for n in names}
    for it in range(warmup + reps):
        e = [_event(torch)]
        rs.chunk_sort(D1, topo, capacity=plan.capacity, out=(plan.chunk_off, plan.chunk_w, plan.chunk_flow, plan.perm), ws=plan.ws_sort)
        e.append(_event(torch))
        rs.lpt_spray(plan.chunk_off, plan.chunk_w, B, topo, out=(plan.rail, plan.S), capacity=plan.capacity, ws=plan.ws_lpt)
        e.append(_event(torch))
        rs.eval(plan.chunk_off, plan.chunk_w, plan.chunk_flow, plan.rail, plan.S, B, topo, out=(plan.R, plan.stats), ws=plan.ws_eval,
                capacity=plan.capacity)
        e.append(_event(torch))
        torch.cuda.synchronize()
        if it >= warmup:
            for i, n in enumerate(names):
                t[n].append(e[i].elapsed_time(e[i + 1]))
    small = [x.clone() for x in (plan.chunk_off, plan.S, plan.R, plan.stats)]
    rail3 = plan.rail.clone()
    for x in (plan.rail, plan.S, plan.R, plan.stats):
        x.zero_()
    one = []
    for it in range(warmup + reps):
        e0 = _event(torch)
        plan.schedule_one_call(D1)
        e1 = _event(torch)
        torch.cuda.synchronize()
        if it >= warmup:
            one.append(e0.elapsed_time(e1))
    assert all(torch.equal(a, b) for a, b in zip(small, (plan.chunk_off, plan.S, plan.R, plan.stats))) and torch.equal(rail3, plan.rail)
    del rail3
    return {n: _median(v) for n, v in t.items()}, _median(one)


def time_chunkwise(rs, torch, plan, B, topo, reps):
    """The plain per-chunk LPT kernel (every chunk through the cross-lane argmin) on the records in `plan`; same outputs."""
    rail2, S2 = torch.empty_like(plan.rail), torch.empty_like(plan.S)
    t = []
    for it in range(1 + reps):
        e0 = _event(torch)
        rs.lpt_spray(plan.chunk_off, plan.chunk_w, B, topo, out=(rail2, S2), chunkwise=True, capacity=plan.capacity, ws=plan.ws_lpt)
        e1 = _event(torch)
        torch.cuda.synchronize()
        if it >= 1:
            t.append(e0.elapsed_time(e1))
    total = int(plan.chunk_off[-1].item())
    assert torch.equal(rail2[:total], plan.rail[:total]) and torch.equal(S2, plan.S)
    del rail2, S2
    return _median(t)


def ratio_stats(np, stats):
    """makespan / lower bound per matrix: max and mean as doubles, the max also as the exact fraction of the two integers."""
    r = stats[:, 0] / np.maximum(stats[:, 3], 1)
    i = int(r.argmax())
    return {"max": float(r.max()), "mean": float(r.mean()), "max_exact": f"{int(stats[i, 0])}/{int(max(stats[i, 3], 1))}", "matrices": int(r.size)}


def exact_mse_over_wmax2(S, wmax):
    """max over matrices and nodes of MSE / w_max^2 with MSE = (1/N) sum_j (L_j - mean)^2 (Algorithm 2 step 6; Theorem 4
    bounds it by w_max^2), in exact integer arithmetic: sum_j (N L_j - T)^2 / (N^3 w_max^2) with T = sum_j L_j."""
    from fractions import Fraction
    best = Fraction(0)
    for b in range(S.shape[0]):
        wm = int(wmax[b])
        if wm == 0:
            continue
        for k in range(S.shape[1]):
            L = [int(x) for x in S[b, k]]
            N, T = len(L), sum(L)
            best = max(best, Fraction(sum((N * x - T) ** 2 for x in L), N ** 3 * wm * wm))
    return float(best)


def cpu_stages_3_5(oracle, np, D1_host, M, N, C, plan_slices):
    """The oracle on a sample of whole matrices: all threads on D1_host, one thread on its first eighth.  plan_slices(n_matrices,
    n_chunks) returns the GPU's (rail[:n_chunks], S, R, stats) of the first n_matrices matrices, to compare."""
    nb = D1_host.shape[0]
    c0 = time.perf_counter()
    off, w, flow, _ = oracle.chunk_sort_batch(D1_host, M, N, C, want_perm=False)
    rail, S = oracle.lpt_batch(off, w, nb, M, N)
    _, R, stats = oracle.eval_batch(off, w, flow, rail, nb, M, N)
    c1 = time.perf_counter()
    n = int(off[-1])
    g_rail, g_S, g_R, g_stats = plan_slices(nb, n)
    same = bool(np.array_equal(g_rail, rail) and np.array_equal(g_S, S) and np.array_equal(g_R, R) and np.array_equal(g_stats, stats))
    del w, flow, rail
    n1 = max(nb // 8, 1)
    allt = oracle.num_threads()
    oracle.set_threads(1)
    s0 = time.perf_counter()
    off1, w1, flow1, _ = oracle.chunk_sort_batch(D1_host[:n1], M, N, C, want_perm=False)
    rail1, _ = oracle.lpt_batch(off1, w1, n1, M, N)
    oracle.eval_batch(off1, w1, flow1, rail1, n1, M, N)
    s1 = time.perf_counter()
    oracle.set_threads(allt)
    return {"value": n / (c1 - c0), "unit": "chunks/s", "cores": allt, "kind": "oracle",
            "sample": f"first {nb} matrices ({nb * M} instances, {n} chunks), stages 3-5, {c1 - c0:.2f} s",
            "matches_gpu": same,
            "single_thread": {"value": int(off1[-1]) / (s1 - s0), "unit": "chunks/s", "cores": 1,
                              "sample": f"first {n1} matrices ({int(off1[-1])} chunks), {s1 - s0:.2f} s"}}


# ------------------------------------------------------------------------------------------------ c1 / c2: resident logits
def bench_resident(cfg, args, rs, W, torch, np):
    dev = "cuda:0"
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
        copy_probe(torch, dev)

    # ---- size the record arrays once (count query), then a plan that allocates nothing per step
    idx0 = rs.route_topk(logits, cfg.k)
    D10 = rs.traffic_matrix(idx0, B, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo)
    total_chunks = rs.chunk_total(D10, topo)
    del idx0, D10
    plan = rs.Plan(topo, B, total_chunks, dev, rows=rows, k=cfg.k, want_perm=True)
    ws_rt = torch.empty(max(rs.route_traffic_workspace_bytes(B, cfg.tokens_per_gpu, cfg.E, cfg.k, topo), 256), dtype=torch.uint8, device=dev)
    ws_tm = torch.empty(max(rs.traffic_matrix_workspace_bytes(B, cfg.tokens_per_gpu, cfg.k, topo), 256), dtype=torch.uint8, device=dev)
    names = {True: ("route_traffic", "schedule"),
             False: ("route_topk", "traffic_matrix", "chunk_sort", "lpt_spray", "eval")}

    def step(fused, events=None):
        marks = []

        def mark():
            if events is not None:
                marks.append(_event(torch))
        mark()
        if fused:
            rs.route_traffic(logits, cfg.k, B, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo,
                             out=(plan.topk_idx, plan.D1), ws=ws_rt); mark()
            plan.schedule_one_call(); mark()
        else:
            rs.route_topk(logits, cfg.k, out=plan.topk_idx); mark()
            rs.traffic_matrix(plan.topk_idx, B, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo, out=plan.D1, ws=ws_tm); mark()
            rs.chunk_sort(plan.D1, topo, capacity=plan.capacity,
                          out=(plan.chunk_off, plan.chunk_w, plan.chunk_flow, plan.perm), ws=plan.ws_sort); mark()
            rs.lpt_spray(plan.chunk_off, plan.chunk_w, B, topo, out=(plan.rail, plan.S), capacity=plan.capacity, ws=plan.ws_lpt); mark()
            rs.eval(plan.chunk_off, plan.chunk_w, plan.chunk_flow, plan.rail, plan.S, B, topo,
                    out=(plan.R, plan.stats), ws=plan.ws_eval, capacity=plan.capacity); mark()
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
        per = {n: [] for n in names[fused]}
        whole = []
        for marks in ev:
            for i, n in enumerate(names[fused]):
                per[n].append(marks[i].elapsed_time(marks[i + 1]))
            whole.append(marks[0].elapsed_time(marks[-1]))
        return (t1 - t0) * 1e3 / args.steps, {n: _median(v) for n, v in per.items()}, _median(whole)

    staged_ms_per_step, staged_ms, staged_median = run(False)
    keep = ("topk_idx", "D1", "chunk_off", "chunk_w", "chunk_flow", "perm", "rail", "S", "R", "stats")
    staged_out = {n: getattr(plan, n).clone() for n in keep}
    for n in keep[2:]:
        getattr(plan, n).fill_(0)
    ms_per_step, stage_ms, step_median = run(True)   # the timed region the headline value comes from
    for n in keep:                                   # both ways give the same bytes
        m = total_chunks if n in ("chunk_w", "chunk_flow", "perm", "rail") else None
        assert torch.equal(staged_out[n][:m], getattr(plan, n)[:m]), n
    del staged_out
    assert int(plan.chunk_off[-1].item()) == total_chunks

    piped_ms = chunkwise_ms = graph_ms = None
    schemes = combine = sweep = placement = None
    stats = plan.stats.cpu().numpy()
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
        outs = (plan.topk_idx, plan.D1, plan.chunk_off, plan.rail, plan.S, plan.R, plan.stats)
        want_g = [t.clone() for t in outs]
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step(True)
        torch.cuda.synchronize()
        for t in outs:
            t.zero_()
        for _ in range(max(args.warmup, 1)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        assert all(torch.equal(a, b) for a, b in zip(want_g, outs))
        del graph, want_g

        chunkwise_ms = time_chunkwise(rs, torch, plan, B, topo, max(min(args.steps, 10), 3))

        # ---- supplementary: the comparison schemes on the same chunk records, and the second all-to-all (transposed traffic)
        def timed(fn):
            fn()
            e0 = _event(torch); fn(); e1 = _event(torch)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1)
        rail2, S2 = torch.empty_like(plan.rail), torch.empty_like(plan.S)
        R2, stats2 = torch.empty_like(plan.R), torch.empty_like(plan.stats)
        schemes = {"lpt": {"makespan_over_lb_" + k_: v for k_, v in ratio_stats(np, stats).items()}}
        for pol in ("nic_direct", "flow_hash", "random_spray", "round_robin"):
            ms = timed(lambda: rs.assign_policy(pol, 1, plan.chunk_off, plan.chunk_w, plan.chunk_flow, B, topo, out=(rail2, S2),
                                                capacity=plan.capacity))
            rs.eval(plan.chunk_off, plan.chunk_w, plan.chunk_flow, rail2, S2, B, topo, out=(R2, stats2), ws=plan.ws_eval, capacity=plan.capacity)
            r2 = ratio_stats(np, stats2.cpu().numpy())
            schemes[pol] = {"makespan_over_lb_max": r2["max"], "makespan_over_lb_mean": r2["mean"], "assign_ms": ms}
        D1T = torch.empty_like(plan.D1)
        tr_ms = timed(lambda: rs.transpose_matrix(plan.D1, topo, out=D1T))
        n_comb = rs.chunk_total(D1T, topo, plan.ws_sort)
        plan_c = rs.Plan(topo, B, n_comb, dev, want_perm=True)
        comb_ms = timed(lambda: plan_c.schedule_one_call(D1T))
        combine = {"transpose_ms": tr_ms, "schedule_ms": comb_ms, "chunks": n_comb,
                   "makespan_over_lb_max": ratio_stats(np, plan_c.stats.cpu().numpy())["max"]}
        del plan_c
        # ---- chunk granularity (Theorem 4): the same traffic matrices cut at other chunk sizes
        sweep = []
        for cb in (16384, 65536, 262144, 1048576, 4194304):
            topo_g = rs.Topo(cfg.M, cfg.N, cb, cfg.rail_bw_Bps)
            n_g = rs.chunk_total(plan.D1, topo_g)
            plan_g = rs.Plan(topo_g, B, n_g, dev, want_perm=True)
            ms_g = timed(lambda: plan_g.schedule_one_call(plan.D1))
            st_g, S_g = plan_g.stats.cpu().numpy(), plan_g.S.cpu().numpy()
            wmax = np.maximum(st_g[:, 5], 1)
            sweep.append({"chunk_bytes": cb, "chunks": n_g, "schedule_ms": ms_g,
                          "makespan_over_lb_max": ratio_stats(np, st_g)["max"],
                          "send_spread_over_wmax_max": float((st_g[:, 7] / wmax).max()),
                          "mse_over_wmax2_max": exact_mse_over_wmax2(S_g, st_g[:, 5])})
            del plan_g
        # ---- expert placement (Section 6.3, sparse against dense): the first R replica groups of the placement table only
        placement = []
        for R_ in sorted({1, 2, max(cfg.replicas // 2, 1), cfg.replicas}):
            eg_R = torch.from_numpy(np.ascontiguousarray(eg_np[:, :R_])).to(dev)
            _, D1_R = rs.route_traffic(logits, cfg.k, B, cfg.tokens_per_gpu, eg_R, cfg.payload_bytes, topo, out=(plan.topk_idx, D1T), ws=ws_rt)
            n_R = rs.chunk_total(D1_R, topo)
            plan_R = rs.Plan(topo, B, n_R, dev, want_perm=True)
            ms_R = timed(lambda: plan_R.schedule_one_call(D1_R))
            st_R = plan_R.stats.cpu().numpy()
            placement.append({"replicas": R_, "gpus_with_experts": R_ * (cfg.E // cfg.experts_per_gpu), "chunks": n_R, "schedule_ms": ms_R,
                              "makespan_over_lb_max": ratio_stats(np, st_R)["max"],
                              "completion_time_us_max": float(st_R[:, 0].max() / cfg.rail_bw_Bps * 1e6)})
            del plan_R
        # leave the plan holding this workload's own outputs again
        rs.route_traffic(logits, cfg.k, B, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo, out=(plan.topk_idx, plan.D1), ws=ws_rt)
        plan.schedule_one_call()
        torch.cuda.synchronize()
        stats = plan.stats.cpu().numpy()

    # ---- rooflines (route_traffic streams the logits once and writes the indices once)
    k1_bytes = rows * (4 * cfg.E + 4 * cfg.k)
    k2_bytes = rows * 4 * cfg.k + 8 * B * G * G
    rt_bytes = k1_bytes + 8 * B * G * G
    sb = stage_bytes(total_chunks, B * cfg.M, topo, True)
    rt_roof = hbm_roofline("route_traffic_kernel (with rt_reduce_kernel, the sum of its slice counts, in the same call)", cfg.name,
                           rt_bytes, stage_ms["route_traffic"], counted=("route_traffic_kernel", "rt_reduce_kernel:one_call"))
    rt_roof["slowest_stage"] = max(stage_ms, key=stage_ms.get)
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
        "timing": "ms_per_step = wall time of the K steps / K; stage_ms and median_step_ms = medians of per-step hipEvent times",
        "median_step_ms": step_median,
        "stage_ms": stage_ms,
        "staged": {"ms_per_step": staged_ms_per_step, "median_step_ms": staged_median, "value": total_chunks / (staged_ms_per_step * 1e-3),
                   "stage_ms": staged_ms,
                   "note": "the same step through the five separate calls (indices written, then read back)",
                   "stage_rooflines": {
                       "route_topk": hbm_roofline("route_topk_kernel", cfg.name, k1_bytes, staged_ms["route_topk"]),
                       "traffic_matrix": hbm_roofline("traffic_matrix_kernel (with the sum of its slice counts)", cfg.name, k2_bytes,
                                                      staged_ms["traffic_matrix"]),
                       **{n: hbm_roofline(STAGE_KERNEL[n], cfg.name, sb[n], staged_ms[n],
                                          note="latency-bound at this size: a few tens of MB through dependent launches")
                          for n in ("chunk_sort", "lpt_spray", "eval")}},
                   "routing_to_traffic_matrix_GBps": (k1_bytes + k2_bytes) / ((staged_ms["route_topk"] + staged_ms["traffic_matrix"]) * 1e-3) / 1e9},
        "two_steps_in_flight": None if piped_ms is None else {
            "ms_per_step": piped_ms, "value": total_chunks / (piped_ms * 1e-3),
            "note": "same two calls per step, consecutive steps alternating between two streams and two sets of outputs"},
        "graph_replay": None if graph_ms is None else {
            "ms_per_step": graph_ms, "value": total_chunks / (graph_ms * 1e-3),
            "note": "the same two calls captured once into a HIP graph and replayed; outputs checked against the eager step"},
        "routing_to_traffic_matrix_GBps": rt_roof["achieved"],
        "routing_frac_of_hbm_peak": rt_roof["frac"],
        "lpt_spray_chunks_per_s": None if chunkwise_ms is None else total_chunks / (chunkwise_ms * 1e-3),
        "lpt_spray_runs_chunks_per_s": total_chunks / (staged_ms["lpt_spray"] * 1e-3),
        "lpt_spray_note": "lpt_spray_chunks_per_s: railsched_lpt_spray_chunkwise, every chunk through the cross-lane argmin (the kernel "
                          "lpt_roofline prices); lpt_spray_runs_chunks_per_s: railsched_lpt_spray, which assigns runs of equal weights in closed form",
        "lpt_roofline": None if chunkwise_ms is None else lpt_alu_roofline(total_chunks, B * cfg.M, cfg.N, chunkwise_ms),
        "lpt_spray_chunkwise_ms": chunkwise_ms,
        "makespan_over_lower_bound": ratio_stats(np, stats),
        "schemes": schemes,
        "granularity_sweep": sweep,
        "placement_sweep": placement,
        "second_all_to_all": combine,
        "completion_time_us_max": float(stats[:, 0].max() / cfg.rail_bw_Bps * 1e6),
        "roofline": rt_roof,
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
            _, R, stats_ = oracle.eval_batch(off, w, flow, rail, layers, cfg.M, cfg.N)
            return off, rail, R, stats_
        c0 = time.perf_counter()
        off_c, rail_c, R_c, stats_c = cpu_path(x, L)
        c1 = time.perf_counter()
        n_c = int(off_c[-1])
        L1 = max(L // 4, 1)                          # the same oracle on one thread, on the first quarter of the sample
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
    del logits, plan
    return out


# ------------------------------------------------------------------------------------------------ c3: resident flow matrices
def bench_flows_resident(cfg, args, rs, W, torch, np):
    """c3: no routing stage; a step is stages 3-5 over all matrices, resident in HBM."""
    dev = "cuda:0"
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes, cfg.rail_bw_Bps)
    B = args.matrices if args.matrices > 0 else cfg.batch
    D1 = W.gen_flow_matrices_device(cfg, dev, first=0, count=B)
    if args.copy_probe:
        copy_probe(torch, dev)
    total = rs.chunk_total(D1, topo)
    plan = rs.Plan(topo, B, total, dev, want_perm=True)
    reps, warmup = max(min(args.steps, 10), 3), min(args.warmup, 2)
    ms, one_ms = time_stages_3_5(rs, torch, plan, D1, topo, B, reps, warmup)
    st = plan.stats.cpu().numpy()
    n_inst = B * cfg.M
    sb = stage_bytes(total, n_inst, topo, True)
    chunkwise_ms = None if args.skip_extras else time_chunkwise(rs, torch, plan, B, topo, 3)
    probe = None if args.skip_extras else write_probe(torch, plan, total)
    if probe is not None:   # the probe overwrote the records: the outputs checked below come from a fresh call
        plan.schedule_one_call(D1)
        torch.cuda.synchronize()
    rec = {
        "metric": "LPT-sprayed chunks/s over stages 3-5 (chunk_sort, lpt_spray, eval, in one call); the workload has no routing stage",
        "value": total / (one_ms * 1e-3), "unit": "chunks/s", "n_gpus": 1, "steps": reps, "warmup": warmup,
        "ms_per_step": one_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64 loads / uint32 weights", "data": "synthetic (seeded lognormal flow matrices)",
        "config": {"workload": f"{cfg.name}: M={cfg.M} nodes x N={cfg.N} rails, {B} of {cfg.batch} matrices of {cfg.G}x{cfg.G}, "
                               f"C={cfg.chunk_bytes} B, p_zero={cfg.p_zero}", "chunks": total, "instances": n_inst, "perm": True},
        "timing": "medians of hipEvent times: railsched_schedule (stages 3-5 in one call) is the step; the three separate calls under `staged`",
        "stage_ms": {"schedule": one_ms},
        "staged": {"ms_per_step": sum(ms.values()), "stage_ms": ms,
                   "stage_rooflines": {n: hbm_roofline(STAGE_KERNEL[n], cfg.name, sb[n], ms[n]) for n in ms}},
        "lpt_spray_chunks_per_s": None if chunkwise_ms is None else total / (chunkwise_ms * 1e-3),
        "lpt_spray_runs_chunks_per_s": total / (ms["lpt_spray"] * 1e-3),
        "lpt_roofline": None if chunkwise_ms is None else lpt_alu_roofline(total, n_inst, cfg.N, chunkwise_ms),
        "lpt_spray_chunkwise_ms": chunkwise_ms,
        "makespan_over_lower_bound": ratio_stats(np, st),
        "roofline": hbm_roofline(STAGE_KERNEL["schedule"], cfg.name, sb["schedule"], one_ms),
        "write_probe": probe,
    }
    if args.cpu_layers != 0:
        import oracle
        nb = min(B, 128)
        off_g = plan.chunk_off.cpu().numpy()

        def slices(nm, n):
            assert int(off_g[nm * cfg.M]) == n
            return plan.rail[:n].cpu().numpy(), plan.S[:nm].cpu().numpy(), plan.R[:nm].cpu().numpy(), plan.stats[:nm].cpu().numpy()
        rec["cpu_baseline"] = cpu_stages_3_5(oracle, np, D1[:nb].cpu().numpy(), cfg.M, cfg.N, cfg.chunk_bytes, slices)
    del D1, plan
    return rec


# ------------------------------------------------------------------------------------------------ c5: one matrix resident at a time
def bench_flows_streamed(cfg, args, rs, W, torch, np):
    """c5: every matrix is ~3.9e9 chunks (35 GB of records), so the matrices go through one at a time: each is generated on
    the device (untimed), then stages 3-5 run on it through railsched_schedule (timed).  Matrix 0 also gets the repeated
    measurement of the three separate calls and of the per-chunk LPT kernel."""
    dev = "cuda:0"
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes, cfg.rail_bw_Bps)
    B = args.matrices if args.matrices > 0 else cfg.batch
    n_inst = cfg.M
    per_matrix, chunks, ratios = [], [], []
    first = None
    plan = None
    for b in range(B):
        D1 = W.gen_flow_matrices_device(cfg, dev, first=b, count=1)
        total = rs.chunk_total(D1, topo)
        if plan is None or plan.capacity < total:
            plan = None
            torch.cuda.empty_cache()
            plan = rs.Plan(topo, 1, total + total // 8, dev, want_perm=False)   # room for the larger matrices to come
        if b == 0:
            if args.copy_probe:
                copy_probe(torch, dev)
            reps, warmup = max(min(args.steps, 10), 3), 1
            ms, one_ms = time_stages_3_5(rs, torch, plan, D1, topo, 1, reps, warmup)
            chunkwise_ms = None if args.skip_extras else time_chunkwise(rs, torch, plan, 1, topo, 2)
            sb = stage_bytes(total, n_inst, topo, False)
            probe = None if args.skip_extras else write_probe(torch, plan, total)
            if probe is not None:
                plan.schedule_one_call(D1)
                torch.cuda.synchronize()
            first = {"chunks": total, "write_probe": probe, "stage_ms": {"schedule": one_ms}, "reps": reps,
                     "staged": {"ms_per_step": sum(ms.values()), "stage_ms": ms,
                                "stage_rooflines": {n: hbm_roofline(STAGE_KERNEL[n], cfg.name, sb[n], ms[n]) for n in ms}},
                     "lpt_spray_chunks_per_s": None if chunkwise_ms is None else total / (chunkwise_ms * 1e-3),
                     "lpt_spray_runs_chunks_per_s": total / (ms["lpt_spray"] * 1e-3),
                     "lpt_roofline": None if chunkwise_ms is None else lpt_alu_roofline(total, n_inst, cfg.N, chunkwise_ms),
                     "lpt_spray_chunkwise_ms": chunkwise_ms,
                     "roofline": hbm_roofline(STAGE_KERNEL["schedule"], cfg.name, sb["schedule"], one_ms)}
            if args.cpu_layers != 0:
                import oracle
                D1_h = D1[0].cpu().numpy()
                c0 = time.perf_counter()
                off_c, S_c, R_c, stats_c = oracle.schedule_matrix_by_node(D1_h, cfg.M, cfg.N, cfg.chunk_bytes)
                c1 = time.perf_counter()
                same = bool(np.array_equal(plan.chunk_off.cpu().numpy(), off_c) and np.array_equal(plan.S[0].cpu().numpy(), S_c)
                            and np.array_equal(plan.R[0].cpu().numpy(), R_c) and np.array_equal(plan.stats[0].cpu().numpy(), stats_c))
                sizes = np.diff(off_c)
                k1 = int(np.argsort(sizes)[len(sizes) // 2])             # one thread: the median instance
                s0 = time.perf_counter()
                cw, cf = oracle.chunk_split(D1_h, cfg.M, cfg.N, cfg.chunk_bytes, k1)
                sw, sf, _ = oracle.sort_desc(cw, cf)
                oracle.lpt(sw, cfg.N)
                s1 = time.perf_counter()
                first["cpu_baseline"] = {"value": int(off_c[-1]) / (c1 - c0), "unit": "chunks/s", "cores": oracle.num_threads(), "kind": "oracle",
                                         "sample": f"matrix 0 of {cfg.batch} (all {cfg.M} instances, {int(off_c[-1])} chunks), stages 3-5 one node "
                                                   f"at a time, {c1 - c0:.2f} s", "matches_gpu": same,
                                         "single_thread": {"value": int(sizes[k1]) / (s1 - s0), "unit": "chunks/s", "cores": 1,
                                                           "sample": f"the median instance ({int(sizes[k1])} chunks), split + sort + LPT, "
                                                                     f"{s1 - s0:.2f} s"}}
                del D1_h, cw, cf, sw, sf
        e0 = _event(torch)
        plan.schedule_one_call(D1)
        e1 = _event(torch)
        torch.cuda.synchronize()
        per_matrix.append(e0.elapsed_time(e1))
        chunks.append(total)
        st = plan.stats.cpu().numpy()
        assert int(st[0, 6]) == total and int(st[0, 0]) >= int(st[0, 3]) > 0
        ratios.append(st[0, 0] / st[0, 3])
        del D1
    step_ms = sum(per_matrix)
    total_all = sum(chunks)
    sb_all = 8 * topo.rails * topo.G * n_inst * B + 9 * total_all
    rec = {
        "metric": "LPT-sprayed chunks/s over stages 3-5 (chunk_sort, lpt_spray, eval, in one call); the workload has no routing stage",
        "value": total_all / (step_ms * 1e-3), "unit": "chunks/s", "n_gpus": 1, "steps": 1, "warmup": 0,
        "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64 loads / uint32 weights", "data": "synthetic (seeded lognormal flow matrices)",
        "config": {"workload": f"{cfg.name}: M={cfg.M} nodes x N={cfg.N} rails, {B} of {cfg.batch} matrices of {cfg.G}x{cfg.G}, one resident at a "
                               f"time, C={cfg.chunk_bytes} B, p_zero={cfg.p_zero}", "chunks": total_all, "instances": n_inst * B, "perm": False},
        "timing": "sum over the matrices of the hipEvent time of railsched_schedule on each (generated on the device between the calls, untimed)",
        "per_matrix_ms": {"median": _median(per_matrix), "min": min(per_matrix), "max": max(per_matrix)},
        "chunks_per_matrix": {"median": _median(chunks), "min": min(chunks), "max": max(chunks)},
        "makespan_over_lower_bound": {"max": float(max(ratios)), "mean": float(sum(ratios) / len(ratios))},
        "roofline": hbm_roofline(STAGE_KERNEL["schedule"], cfg.name, sb_all / B, step_ms / B,
                                 note="average over the matrices: algorithmic bytes and time per matrix"),
        "matrix_0": first,
    }
    if first and "cpu_baseline" in first:
        rec["cpu_baseline"] = first["cpu_baseline"]
    del plan
    return rec


# ------------------------------------------------------------------------------------------------ c4: logits streamed layer by layer
def bench_streamed(cfg, args, rs, W, torch, np):
    """c4: 244 GiB of logits in all, so each layer's 4 GiB is generated into HBM (untimed), stages 1-2 are timed on it,
    and stages 3-5 run once over the 61 matrices."""
    dev = "cuda:0"
    topo = rs.Topo(cfg.M, cfg.N, cfg.chunk_bytes, cfg.rail_bw_Bps)
    B, G = (args.layers if args.layers > 0 else cfg.batch), cfg.G
    eg_np = W.expert_gpu_table(cfg)
    expert_gpu = torch.from_numpy(eg_np).to(dev)
    D1 = torch.empty((B, G, G), dtype=torch.int64, device=dev)
    idx = torch.empty((cfg.rows_per_layer, cfg.k), dtype=torch.int32, device=dev)
    ws_tm = torch.empty(max(rs.traffic_matrix_workspace_bytes(1, cfg.tokens_per_gpu, cfg.k, topo), 256), dtype=torch.uint8, device=dev)
    ws_rt = torch.empty(max(rs.route_traffic_workspace_bytes(1, cfg.tokens_per_gpu, cfg.E, cfg.k, topo), 256), dtype=torch.uint8, device=dev)
    D1_one = torch.empty((1, G, G), dtype=torch.int64, device=dev)
    idx_one = torch.empty_like(idx)
    t1, t2, t12, t12n = [], [], [], []
    keep_logits = []
    for b in range(B):
        lg = W.gen_logits(cfg, b, device=dev)
        if b == 0:
            if args.copy_probe:
                copy_probe(torch, dev)
            rs.route_topk(lg, cfg.k, out=idx)           # warm-up launches
            rs.route_traffic(lg, cfg.k, 1, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo, out=(idx_one, D1_one), ws=ws_rt)
        e0 = _event(torch)
        rs.route_topk(lg, cfg.k, out=idx)
        e1 = _event(torch)
        rs.traffic_matrix(idx, 1, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo, out=D1[b:b + 1], ws=ws_tm)
        e2 = _event(torch)
        rs.route_traffic(lg, cfg.k, 1, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo, out=(idx_one, D1_one), ws=ws_rt)
        e3 = _event(torch)
        torch.cuda.synchronize()
        t1.append(e0.elapsed_time(e1)); t2.append(e1.elapsed_time(e2)); t12.append(e2.elapsed_time(e3))
        assert torch.equal(D1_one[0], D1[b]) and torch.equal(idx_one, idx)
        if not args.skip_extras:                    # the same call without the indices: one pass over the logits
            e4 = _event(torch)
            rs.route_traffic(lg, cfg.k, 1, cfg.tokens_per_gpu, expert_gpu, cfg.payload_bytes, topo, out=(None, D1_one), ws=ws_rt)
            e5 = _event(torch)
            torch.cuda.synchronize()
            t12n.append(e4.elapsed_time(e5))
            assert torch.equal(D1_one[0], D1[b])
        if b < 2 and args.cpu_layers != 0:
            keep_logits.append(lg.cpu().numpy())
        del lg
    del idx, idx_one, D1_one
    total = rs.chunk_total(D1, topo)
    plan = rs.Plan(topo, B, total, dev, want_perm=True)
    reps, warmup = max(min(args.steps, 10), 3), min(args.warmup, 2)
    ms3, one_ms = time_stages_3_5(rs, torch, plan, D1, topo, B, reps, warmup)
    chunkwise_ms = None if args.skip_extras else time_chunkwise(rs, torch, plan, B, topo, 3)
    ms = {"route_traffic": sum(t12), "schedule": one_ms}
    step_ms = sum(ms.values())
    rows = B * cfg.rows_per_layer
    k1_bytes = cfg.rows_per_layer * (4 * cfg.E + 4 * cfg.k)             # per layer = per launch
    k2_bytes = cfg.rows_per_layer * 4 * cfg.k + 8 * G * G
    rt_bytes = k1_bytes + 8 * G * G
    st = plan.stats.cpu().numpy()
    n_inst = B * cfg.M
    sb = stage_bytes(total, n_inst, topo, True)
    rec = {
        "metric": "LPT-sprayed chunks/s over the whole path (route_topk, traffic_matrix, chunk_sort, lpt_spray, eval; stages 1-2 and 3-5 fused into two calls)",
        "value": total / (step_ms * 1e-3), "unit": "chunks/s", "n_gpus": 1, "steps": 1, "warmup": 1,
        "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64 loads / uint32 weights / fp32 compare-only", "data": "synthetic (seeded counter-based logits, Zipf expert bias)",
        "config": {"workload": f"{cfg.name}: DeepSeek-V3-shaped, M={cfg.M} nodes x N={cfg.N} rails, E={cfg.E} top-{cfg.k}, {cfg.tokens_per_gpu} "
                               f"tokens/GPU x {cfg.payload_bytes} B, C={cfg.chunk_bytes} B, {B} of {cfg.batch} matrices of {G}x{G}", "rows": rows,
                   "chunks": total, "instances": n_inst},
        "timing": "sum of hipEvent times: railsched_route_traffic once per layer (logits regenerated between layers, untimed), "
                  "railsched_schedule over all matrices (median of the repetitions)",
        "stage_ms": ms,
        "per_layer_ms": {"route_traffic": _median(t12), "route_topk": _median(t1), "traffic_matrix": _median(t2),
                         "route_traffic_without_indices": _median(t12n)},
        "staged": {"ms_per_step": sum(t1) + sum(t2) + sum(ms3.values()),
                   "stage_ms": {"route_topk": sum(t1), "traffic_matrix": sum(t2), **ms3},
                   "stage_rooflines": {
                       "route_topk": hbm_roofline("route_topk_insert_kernel", cfg.name, k1_bytes, _median(t1)),
                       "traffic_matrix": hbm_roofline("traffic_matrix_kernel (with the sum of its slice counts)", cfg.name, k2_bytes, _median(t2)),
                       **{n: hbm_roofline(STAGE_KERNEL[n], cfg.name, sb[n], ms3[n]) for n in ms3}},
                   "routing_to_traffic_matrix_GBps": (k1_bytes + k2_bytes) / ((_median(t1) + _median(t2)) * 1e-3) / 1e9},
        "routing_to_traffic_matrix_GBps": rt_bytes / (_median(t12) * 1e-3) / 1e9,
        "routing_frac_of_hbm_peak": rt_bytes / (_median(t12) * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "schedule_roofline": hbm_roofline(STAGE_KERNEL["schedule"], cfg.name, sb["schedule"], one_ms),
        "lpt_spray_chunks_per_s": None if chunkwise_ms is None else total / (chunkwise_ms * 1e-3),
        "lpt_spray_runs_chunks_per_s": total / (ms3["lpt_spray"] * 1e-3),
        "lpt_roofline": None if chunkwise_ms is None else lpt_alu_roofline(total, n_inst, cfg.N, chunkwise_ms),
        "lpt_spray_chunkwise_ms": chunkwise_ms,
        "makespan_over_lower_bound": ratio_stats(np, st),
        "roofline": hbm_roofline("route_topk_insert_kernel (railsched_route_traffic on one layer)", cfg.name, rt_bytes, _median(t12),
                                 note="per layer: median over the layers"),
    }
    if keep_logits:
        import oracle
        x = np.concatenate(keep_logits)
        L = len(keep_logits)
        keep_logits.clear()
        c0 = time.perf_counter()
        idx_c = oracle.route_topk(x, cfg.k)
        ctop = time.perf_counter()
        D1c = oracle.traffic_matrix(idx_c, L, cfg.tokens_per_gpu, eg_np, cfg.payload_bytes, cfg.M, cfg.N)
        off, w, flow, _ = oracle.chunk_sort_batch(D1c, cfg.M, cfg.N, cfg.chunk_bytes, want_perm=False)
        rail, S = oracle.lpt_batch(off, w, L, cfg.M, cfg.N)
        _, R, stats_c = oracle.eval_batch(off, w, flow, rail, L, cfg.M, cfg.N)
        c1 = time.perf_counter()
        n_c = int(off[-1])
        same = bool(np.array_equal(D1[:L].cpu().numpy(), D1c) and np.array_equal(plan.rail[:n_c].cpu().numpy(), rail)
                    and np.array_equal(plan.S[:L].cpu().numpy(), S) and np.array_equal(plan.R[:L].cpu().numpy(), R)
                    and np.array_equal(plan.stats[:L].cpu().numpy(), stats_c))
        r1 = cfg.rows_per_layer // 16                                    # one thread: stage 1 on a sixteenth of a layer
        allt = oracle.num_threads()
        oracle.set_threads(1)
        s0 = time.perf_counter()
        oracle.route_topk(x[:r1], cfg.k)
        s1 = time.perf_counter()
        oracle.set_threads(allt)
        rec["cpu_baseline"] = {"value": n_c / (c1 - c0), "unit": "chunks/s", "cores": allt, "kind": "oracle",
                               "sample": f"first {L} of {cfg.batch} layers ({L * cfg.rows_per_layer} rows, {n_c} chunks), whole path, "
                                         f"{c1 - c0:.2f} s, of which stage 1 {ctop - c0:.2f} s", "matches_gpu": same,
                               "single_thread": {"value": r1 / (s1 - s0), "unit": "rows/s", "cores": 1,
                                                 "sample": f"stage 1 (top-{cfg.k} of {cfg.E}) on {r1} rows, {s1 - s0:.2f} s"}}
        del x
    del D1, plan
    return rec


def run_config(name, args, rs, W, torch, np):
    cfg = W.get_config(name)
    if cfg.kind == "flows":
        return bench_flows_resident(cfg, args, rs, W, torch, np) if cfg.G <= 256 else bench_flows_streamed(cfg, args, rs, W, torch, np)
    if cfg.rows_per_layer * cfg.batch * cfg.E * 4 > 64 << 30:
        return bench_streamed(cfg, args, rs, W, torch, np)
    return bench_resident(cfg, args, rs, W, torch, np)


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _name_the_cpu(rec, model):
    """Every cpu_baseline object says which CPU the oracle ran on and how the record's GPU rate compares (same unit)."""
    if isinstance(rec, dict):
        for k, v in rec.items():
            if k == "cpu_baseline" and isinstance(v, dict):
                v["cpu_model"] = model
                v["host_cpus"] = os.cpu_count()
                gpu = rec.get("value") if rec.get("unit") == v.get("unit") else None
                if gpu and v.get("value"):
                    v["gpu_over_cpu"] = gpu / v["value"]
                    one = v.get("single_thread")
                    if isinstance(one, dict) and one.get("value") and one.get("unit") == v.get("unit"):
                        one["gpu_over_cpu"] = gpu / one["value"]
            else:
                _name_the_cpu(v, model)


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library runs on exactly one GPU (the rails and the other GPUs are simulated "
              "arithmetically); --gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import gc
    import numpy as np
    import torch
    import workloads as W
    import paper_2510_19262_amd as rs

    rs.load()                                       # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    streams = measure_streams(torch, "cuda:0")
    if args.config != "all":
        out = run_config(args.config, args, rs, W, torch, np)
        out["hbm_measured"] = streams
        _name_the_cpu(out, _cpu_model())
        print(json.dumps(out))
        return
    out = run_config("c2", args, rs, W, torch, np)
    out["hbm_measured"] = streams
    out["workloads"] = {}
    for name in ("c3", "c4", "c5"):
        gc.collect()
        torch.cuda.empty_cache()
        t0 = time.perf_counter()
        try:
            rec = run_config(name, args, rs, W, torch, np)
        except Exception as exc:                    # the headline stands on its own: a sub-record that fails says so
            rec = {"error": f"{type(exc).__name__}: {exc}"}
        rec["wall_s"] = time.perf_counter() - t0
        out["workloads"][name] = rec
        print(f"bench: {name} done in {rec['wall_s']:.1f} s", file=sys.stderr, flush=True)
    _name_the_cpu(out, _cpu_model())
    print(json.dumps(out))


if __name__ == "__main__":
    main()
