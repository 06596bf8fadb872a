#!/usr/bin/env python3
"""Benchmark of the bubble-harvesting hot path on one MI355X.

One step = one pipeline epoch of the emulated stage (its FP/BP GEMM bursts and the waits that stand for the
other stages) with the PageRank side task harvesting every bubble.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg5]

The headline workload is the largest configuration (cfg5: GPipe p=16 m=16 stage 8, R-MAT 2^26 vertices / 2^30
edges, 100 iterations, 40 GB cap); `per_config` carries the same figures, from shorter runs, for cfg2 - cfg4.
Every configuration's harvested ranks are compared with the fp64 CPU oracle in the same invocation.
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

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
PARITY_TOL_ABS = 1e-5        # max |gpu - oracle| (fp32 ranks against the fp64 oracle)
PARITY_TOL_REL = 1e-4        # the same relative to the rank, over ranks above 1/V
KERNEL_SOURCES = ("paper_2409_06941_amd/csrc/pagerank.hip", "paper_2409_06941_amd/csrc/pagerank_prep.hip",
                  "paper_2409_06941_amd/csrc/pr_layout.h")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_sources_sha256():
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def traffic_from_profiles(cfg_name):
    """HBM-side bytes one iteration (k_scatter + k_gather) moves, from the FETCH_SIZE / WRITE_SIZE summary kept under
    profiles/ for this configuration; None if there is none or if the kernels have changed since it was taken."""
    path = os.path.join(ROOT, "profiles", "pagerank_iteration_%s_hbm_traffic_counters.txt" % cfg_name)
    if not os.path.exists(path):
        return None, "no counter summary for %s under profiles/" % cfg_name
    text = open(path).read()
    sha = re.search(r"kernel_sources_sha256:\s*([0-9a-f]{64})", text)
    val = re.search(r"traffic_bytes_per_iteration:\s*([0-9.eE+]+)", text)
    if not sha or not val:
        return None, "summary has no machine-readable figures"
    if sha.group(1) != kernel_sources_sha256():
        return None, "the kernels have changed since the counters were taken"
    return float(val.group(1)), os.path.relpath(path, ROOT)


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def stage_load(cfg, stage_stream):
    """The stage's load and its declared FP/BP durations (medians of timed bursts)."""
    import torch

    import paper_2409_06941_amd as fr
    ws = None
    if cfg.load is not None:
        L = cfg.load
        need = fr.Load.fr_load_workspace_bytes(fr.FR_LOAD_GPT, L.layers, L.hidden, L.ffn, L.tokens)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        load = fr.Load(fr.FR_LOAD_GPT, L.layers, L.hidden, L.ffn, L.tokens, workspace=ws, seed=cfg.seed, stream=stage_stream)
        fp_flops, bp_flops = load.fr_load_flops()

        def timed(fn, n):
            out = []
            for _ in range(n):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                with torch.cuda.stream(stage_stream):
                    a.record(stage_stream)
                    fn(stage_stream)
                    b.record(stage_stream)
                b.synchronize()
                out.append(a.elapsed_time(b) * 1e6)
            return out
        timed(load.fr_load_fp, 3); timed(load.fr_load_bp, 3)
        f_ns = int(statistics.median(timed(load.fr_load_fp, 10)))
        b_ns = int(statistics.median(timed(load.fr_load_bp, 10)))
    else:
        load = fr.Load(fr.FR_LOAD_BUSYWAIT, fp_ns=cfg.busy_fp_ns, bp_ns=cfg.busy_bp_ns)
        fp_flops = bp_flops = 0
        f_ns, b_ns = cfg.busy_fp_ns, cfg.busy_bp_ns
    return load, ws, f_ns, b_ns, fp_flops, bp_flops


def run_config(name, steps, warmup, args, headline):
    """Calibrates, harvests `steps` timed epochs of configuration `name` and returns the result object."""
    import numpy as np
    import torch

    import paper_2409_06941_amd as fr
    from workloads import configs

    cfg = configs.by_name(name)
    t_setup = time.time()
    g = cfg.build_graph()
    V, E, K = g.n_vertices, g.n_edges, cfg.iterations
    log("graph %s: V=%d E=%d built in %.1fs" % (cfg.name, V, E, time.time() - t_setup))
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    rp, col, od = dev(g.row_ptr), dev(g.col), dev(g.out_degree)
    ranks = torch.zeros(V, dtype=torch.float32, device="cuda")
    stage_stream = torch.cuda.Stream()
    cu_count = cfg.cu_count if cfg.cu_count < 256 else 0

    load, ws, f_ns, b_ns, fp_flops, bp_flops = stage_load(cfg, stage_stream)
    log("stage load: f=%.3f ms b=%.3f ms" % (f_ns / 1e6, b_ns / 1e6))

    # ---- side-task profile: per-step costs from a few standalone iterations (the paper's side-task profiler)
    side_probe = fr.Context(device_id=0, cu_count=cu_count)
    cal_iters = 5
    cal = fr.PageRankTask(V, E, rp, col, od, ranks, damping=cfg.damping, iterations=cal_iters)
    t_init = time.time()
    cal.fr_pagerank_run_standalone(0, side_probe.fr_side_stream(), 0, want_phase_ns=False)      # init + warm
    t_init = time.time() - t_init
    ph = cal.fr_pagerank_run_standalone(0, side_probe.fr_side_stream(), 0, want_phase_ns=True)
    info = cal.fr_pagerank_info()
    n_finish_tiles = cal.fr_pagerank_tiles(fr.FR_PR_SEG_FINISH)
    # multiplicands of the task's cost formulas, summed over a sweep
    gather_weight = sum(cal.fr_pagerank_tile_weights(fr.FR_PR_SEG_GATHER))
    scatter_weight = sum(cal.fr_pagerank_tile_weights(fr.FR_PR_SEG_SCATTER))
    tile_cost_spread = []
    for kind in range(4):
        c = cal.fr_pagerank_tile_costs(kind)
        tile_cost_spread.append(max(c) * len(c) / max(1, sum(c)))      # heaviest tile / mean tile
    cal.fr_pagerank_destroy()
    if args.profile_standalone:
        # for counter and trace runs: every k_scatter / k_gather dispatch up to here is a whole sweep of the iteration
        print(json.dumps({"config": cfg.name, "standalone_us": {"k_scatter": ph[1] / cal_iters / 1e3, "k_gather": ph[2] / cal_iters / 1e3},
                          "whole_sweeps_per_kernel": 2 * cal_iters, "kernel_sources_sha256": kernel_sources_sha256(),
                          "algorithmic_bytes_per_iteration": 4.0 * E + 24.0 * V + 4.0,
                          "layout": {"messages": info.messages, "messages_per_edge": info.messages / max(1, E),
                                     "partial_rows": info.partial_rows, "nonempty_ranges": info.nonempty_ranges,
                                     "gather_tiles": info.gather_tiles, "scatter_tiles": info.scatter_tiles}}))
        side_probe.fr_destroy()
        sys.exit(0)
    # shortest steps: one iteration launched one tile at a time; a launch of a few tiles takes about as long as
    # one tile alone, which the additive tile costs cannot express (min_step_ns of the task's cost model)
    one = fr.PageRankTask(V, E, rp, col, od, ranks, damping=cfg.damping, iterations=1)
    ph1 = one.fr_pagerank_run_standalone(0, side_probe.fr_side_stream(), 1, want_phase_ns=True)
    n_tiles_kind = [one.fr_pagerank_tiles(k) for k in range(4)]
    one.fr_pagerank_destroy()
    # (mean over the tiles, scaled to the heaviest tile by the default cost model's spread)
    one_tile_ns = [ph1[k] / max(1, n_tiles_kind[k]) * tile_cost_spread[k] for k in range(4)]
    side_probe.fr_destroy()
    M = max(1, info.messages)
    v_ns, s_ns, g_ns, h_ns = ph[0], ph[1] / cal_iters, ph[2] / cal_iters, ph[3]      # V0 and H run once per run

    def rates(v_ns, s_ns, g_ns, h_ns, derate):
        """Femtosecond rates of the task's cost model from per-segment times (ns) of one iteration."""
        pv = max(1, int(v_ns * 1e6 * derate / V))
        pm = max(1, int(s_ns * 1e6 * derate / (M + scatter_weight)))
        pe = max(1, int(2 * g_ns * 1e6 * derate / max(1, gather_weight)))
        return dict(fs_per_vertex=pv, fs_per_message=pm, fs_per_edge=pe,
                    finish_tile_ns=max(1, int(h_ns * derate / n_finish_tiles)),
                    min_step_ns=[int(derate * x) for x in one_tile_ns])
    log("layout: M/E=%.3f, %d ranges (%d with edges, %d merged), %d gather tiles, %d scatter tiles, %d / %d workgroups a launch, init+first run %.2fs" %
        (info.messages / max(1, E), info.ranges, info.nonempty_ranges, info.merged_ranges, info.gather_tiles,
         info.scatter_tiles, info.gather_slots, info.scatter_slots, t_init))
    log("standalone per iteration: scatter %.1f us, gather %.1f us (once per run: first vertex pass %.1f us, finish %.1f us)" %
        (s_ns / 1e3, g_ns / 1e3, v_ns / 1e3, h_ns / 1e3))
    log("shortest steps (one tile per launch): vertex %.1f us, scatter %.1f us, gather %.1f us, finish %.1f us" %
        tuple(x / 1e3 for x in one_tile_ns))
    standalone_iter_ns = s_ns + g_ns

    # ---- runtime, task, stage
    mem_cap = cfg.mem_cap_bytes if cfg.mem_cap_bytes else (64 << 30)
    kind = fr.FR_SCHED_1F1B if cfg.schedule == "1f1b" else fr.FR_SCHED_GPIPE
    chunks = 0
    if args.interleave > 1:
        # the same stage under interleaved 1F1B with that many model chunks: an operation is one chunk's share of
        # the burst, the bubbles add up to 1 / chunks of the plain schedule's, in more and shorter windows
        if cfg.schedule != "1f1b" or cfg.m % cfg.p or (cfg.load and cfg.load.layers % args.interleave):
            raise SystemExit("bench.py: --interleave needs a 1F1B configuration with m a multiple of p and layers a multiple of the chunks")
        kind, chunks = fr.FR_SCHED_INTERLEAVED, args.interleave
        f_ns, b_ns = f_ns // chunks, b_ns // chunks
    stage = fr.Stage(kind, cfg.p, cfg.m, cfg.stage, f_ns, b_ns, load, stage_stream, chunks=chunks)
    _, ideal_epoch_ns, _ = stage.fr_stage_ops()
    n_segs = 2 * K + 2
    seg_kind = lambda g: (fr.FR_PR_SEG_VERTEX if g == 0 else fr.FR_PR_SEG_FINISH if g == n_segs - 1
                          else fr.FR_PR_SEG_SCATTER + ((g - 1) & 1))
    # the guard also has to cover what a step of a round or less may take beyond its model (its tiles run side by
    # side at a rate the additive costs do not describe): a quarter of the heaviest tile's time alone
    guard_ns = max(args.guard_ns if args.guard_ns else (60_000 if args.device_gate else 150_000),
                   int(0.25 * max(one_tile_ns[1], one_tile_ns[2])))

    def start_task(launch_cost_ns, model, time_steps, adapt=0):
        ctx = fr.Context(device_id=0, cu_count=cu_count,
                         mem_available_bytes=mem_cap + 1, guard_ns=guard_ns, launch_cost_ns=launch_cost_ns,
                         max_chunk_ns=0, max_inflight=32, time_steps=time_steps, event_log_capacity=1 << 18,
                         device_gate=args.device_gate, gate_guard_ns=args.gate_guard_ns, adapt_costs=adapt)
        task = fr.PageRankTask(V, E, rp, col, od, ranks, damping=cfg.damping, iterations=K, max_runs=0,
                               mem_limit_bytes=mem_cap, **model)
        tid = ctx.fr_task_register(task.ops, task.user, task.profile)
        ctx.fr_bubble_begin(fr.fr_now_ns(), 5_000_000_000)          # a long first bubble for InitSideTask
        t_end = time.time() + 60
        while ctx.fr_query_progress(tid).state == fr.FR_CREATED and time.time() < t_end:
            time.sleep(0.001)
        ctx.fr_bubble_end()
        return ctx, task, tid

    # Second profiling pass, in place: an epoch shows what a step costs inside real bubbles, launch gaps included.
    # It is done twice: first with the standalone model, generously derated, then with what the first pass
    # measured - a bubble's first steps run some percent slower than its later ones, so a pass that plans fewer
    # steps per bubble than the timed epochs will measures a slower average than theirs.  The final model is the
    # second pass's cost plus a small margin.
    ts = max(1, args.time_steps)
    standalone = (v_ns, s_ns, g_ns, h_ns)
    n_untimed = 3 if ideal_epoch_ns < 500_000_000 else 1     # right after a start the steps run a few percent slower
    n_tiles = None

    def in_bubble_ratio(launch_cost_ns, model):
        nonlocal n_tiles
        ctx, task, tid = start_task(launch_cost_ns, model, ts)
        for _ in range(n_untimed):
            stage.fr_stage_run_epoch(ctx)
        time.sleep(0.02)
        ctx.fr_event_log_clear()
        stage.fr_stage_run_epoch(ctx)
        time.sleep(0.02)
        n_tiles = [task.fr_pagerank_tiles(k) for k in range(4)]
        # timing groups made of whole sweeps only: measured time against what the standalone profile says they cost
        ratios, group = [], []
        for e in ctx.fr_event_log(1 << 18):
            if e.kind != fr.FR_EV_CHUNK:
                group = []
                continue
            if group and group[-1].bubble != e.bubble:
                group = []
            group.append(e)
            if e.measured_ns > 0:
                if all(x.tile0 == 0 and x.tile1 == n_tiles[seg_kind(x.segment)] for x in group) and \
                   all(seg_kind(x.segment) in (fr.FR_PR_SEG_SCATTER, fr.FR_PR_SEG_GATHER) for x in group) and len(group) == ts:
                    ratios.append(e.measured_ns / sum(standalone[seg_kind(x.segment)] for x in group))
                group = []
        ctx.fr_task_stop(tid); task.fr_pagerank_destroy(); ctx.fr_destroy()
        return ratios
    ratios = in_bubble_ratio(8_000, rates(v_ns, s_ns, g_ns, h_ns, args.derate))
    first_pass = statistics.median(ratios) if ratios else args.derate
    one_tile_standalone = list(one_tile_ns)
    one_tile_ns = [x * first_pass for x in one_tile_standalone]
    ratios = in_bubble_ratio(0, rates(*[x * first_pass for x in standalone], args.margin)) or ratios
    in_bubble = statistics.median(ratios) if ratios else first_pass
    insitu = [x * in_bubble for x in standalone]
    log("in-bubble step times = standalone x %.3f (first pass %.3f; %d timing groups of %d whole sweeps): scatter %.1f us, gather %.1f us" %
        (in_bubble, first_pass, len(ratios), ts, insitu[1] / 1e3, insitu[2] / 1e3))
    if len(ratios) >= 2:
        log("  group ratios min %.3f quartiles %.3f %.3f %.3f max %.3f" % ((min(ratios),) + tuple(statistics.quantiles(ratios, n=4)) + (max(ratios),)))
    one_tile_ns = [x * in_bubble for x in one_tile_standalone]
    ctx, task, tid = start_task(0, rates(*insitu, args.margin), ts, args.adapt_costs)     # the measured group times already hold the launch gaps

    # ---- epochs.  Three arms: with the side task (A), with idle bubbles (B), and with the bubbles filled by
    # register-only arithmetic on the side stream (C: the GPU stays as busy as in A but no memory traffic competes
    # with the stage).  Blocks alternate B a A C a A B C, `a` an untimed epoch with the side task (its first bubbles
    # after a pause run some percent slower), so that drift of clocks and temperature hits all arms alike.
    stage.fr_stage_set_filler(ctx.fr_side_stream(), 4 * max(8, cfg.cu_count), guard_ns)
    ops, _, _ = stage.fr_stage_ops()
    after_bubble = [op.bubble_before_ns > 0 for op in ops]

    def epochs(n, arm):
        out = []
        for _ in range(n):
            if arm == "C":
                stage.fr_stage_set_filler(ctx.fr_side_stream(), 4 * max(8, cfg.cu_count), guard_ns)
            elif arm == "B":
                stage.fr_stage_set_filler(None, 0, 0)
            r = stage.fr_stage_run_epoch(ctx if arm == "A" else None)
            out.append((r, stage.fr_stage_op_times()))
        return out

    for _ in range(max(1, warmup)):
        epochs(1, "A")                           # includes nothing of the task's initialisation: that had its own bubble
    torch.cuda.synchronize()
    half = [steps - steps // 2, steps // 2]
    # (the arms without the side task get a quarter of the timed epochs per block, but no more than what keeps the
    # whole default run within a few minutes when the epochs are seconds long)
    nb = max(1, steps // 4)
    if ideal_epoch_ns >= 500_000_000:
        nb = min(nb, 2)
    with_task, idle, busy, events = [], [], [], []
    p_edges = 0
    prog0 = ctx.fr_query_progress(tid)
    wall_s = 0.0
    for block in range(2):
        (idle if block == 0 else busy).extend(epochs(nb, "B" if block == 0 else "C"))
        if half[block] == 0:
            continue
        epochs(1, "A")
        time.sleep(0.02)
        ctx.fr_event_log_clear()
        p0 = ctx.fr_query_progress(tid)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with_task.extend(epochs(half[block], "A"))
        torch.cuda.synchronize()
        wall_s += time.perf_counter() - t0
        time.sleep(0.05)
        events.extend(ctx.fr_event_log(1 << 18))
        p_edges += ctx.fr_query_progress(tid).work_units_done - p0.work_units_done
    idle.extend(epochs(nb, "B"))
    busy.extend(epochs(nb, "C"))
    prog1 = ctx.fr_query_progress(tid)
    ctx.fr_task_stop(tid)
    edges = p_edges

    if args.dump_events and headline:
        with open(args.dump_events, "w") as fh:
            for r, _ in with_task:
                fh.write(json.dumps({"epoch_ns": r.epoch_ns, "busy_ns": r.busy_ns, "bubble_ns": r.bubble_ns,
                                     "n_bubbles": r.n_bubbles, "overruns": r.overruns}) + "\n")
            for e in events:
                fh.write(json.dumps({"kind": e.kind, "bubble": e.bubble, "run": e.run, "segment": e.segment,
                                     "tile0": e.tile0, "tile1": e.tile1, "modelled_ns": e.modelled_ns,
                                     "measured_ns": e.measured_ns, "t_host_ns": e.t_host_ns}) + "\n")
    bubble_ns = sum(r.bubble_ns for r, _ in with_task)
    chunk_ns = sum(e.measured_ns for e in events if e.kind == fr.FR_EV_CHUNK)
    idle_ns = sum(e.modelled_ns for e in events if e.kind == fr.FR_EV_IDLE)
    # Steps are timed in groups (HIP events on the side stream around every --time-steps consecutive steps of a bubble);
    # a group's time sits on its last step's record.  Only groups that have resolved count, with all their steps.
    timed, group = [], []
    for e in events:
        if e.kind != fr.FR_EV_CHUNK:
            continue
        if group and group[-1].bubble != e.bubble:
            group = []                               # a group never spans two bubbles
        group.append(e)
        if e.measured_ns > 0:
            timed += group
            group = []
    # (with the device gate a step that was refused as a whole keeps its CHUNK record next to a REFUSED record of the
    # same tiles: it did no work, and what time its kernel took stays in its group)
    key = lambda e: (e.bubble, e.run, e.segment, e.tile0, e.tile1)
    refused_whole = {key(e) for e in events if e.kind == fr.FR_EV_REFUSED}
    timed = [e for e in timed if key(e) not in refused_whole or e.measured_ns > 0]
    worked = lambda e: key(e) not in refused_whole
    per_kind_n = [sum(1 for e in timed if worked(e) and seg_kind(e.segment) == k) for k in range(4)]
    timed_edges = sum(e.work_units for e in timed if worked(e))
    # One iteration = one scatter + one gather sweep and moves 4E + 24V + 4 algorithmic bytes (col entries, row starts, one
    # compulsory read of every contribution, the rank write, and the vertex pass); iterations done = edges / E.
    iters_done = timed_edges / E
    pull_ns = sum(e.measured_ns for e in timed)
    iter_bytes = 4.0 * E + 24.0 * V + 4.0
    pull_gbs = iters_done * iter_bytes / pull_ns if pull_ns else 0.0

    def arm_stats(arm):
        ep = [r.epoch_ns for r, _ in arm]
        bz = [r.busy_ns for r, _ in arm]
        first = [t for _, times in arm for t, ab in zip(times, after_bubble) if ab]
        other = [t for _, times in arm for t, ab in zip(times, after_bubble) if not ab]
        return dict(epoch_ms_mean=statistics.mean(ep) / 1e6, epoch_ms_min_med_max=[min(ep) / 1e6, statistics.median(ep) / 1e6, max(ep) / 1e6],
                    busy_ms_mean=statistics.mean(bz) / 1e6, epochs=len(ep),
                    burst_ms_first_after_bubble=(statistics.mean(first) / 1e6) if first else None,
                    burst_ms_others=(statistics.mean(other) / 1e6) if other else None)
    sa, sb, sc = arm_stats(with_task), arm_stats(idle), arm_stats(busy)
    pct = lambda x, y: 100.0 * (x - y) / y if (x is not None and y) else None

    # context for the roofline: what a plain device-to-device copy of 1 GiB moves on this GPU (read + write)
    cp_src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
    cp_dst = torch.empty_like(cp_src)
    cp_dst.copy_(cp_src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(10):
        cp_dst.copy_(cp_src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbs = 10 * 2.0 * cp_src.numel() * 4 / (ev0.elapsed_time(ev1) * 1e6)
    del cp_src, cp_dst

    traffic, traffic_note = traffic_from_profiles(cfg.name)
    traffic_gbs = (traffic * iters_done / pull_ns) if (traffic and pull_ns) else None
    out = {
        "metric": "side-task GTEPS harvested in bubbles",
        "value": edges / bubble_ns if bubble_ns else 0.0,
        "unit": "GTEPS",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": sa["epoch_ms_mean"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %s p=%d m=%d stage=%d; PageRank on %s 2^%d vertices, %d edges, %d iterations, seed %d"
                   % (cfg.name, cfg.schedule, cfg.p, cfg.m, cfg.stage, cfg.graph, cfg.scale, E, K, cfg.seed),
                   "stage_load": ("bf16 GEMM bursts: %d GPT layers h=%d ffn=%d tokens=%d" %
                                  (cfg.load.layers, cfg.load.hidden, cfg.load.ffn, cfg.load.tokens)) if cfg.load else "busy-wait",
                   "schedule": ("interleaved 1F1B, %d chunks" % chunks) if chunks else cfg.schedule,
                   "f_ms": f_ns / 1e6, "b_ms": b_ns / 1e6, "cu_count": cfg.cu_count,
                   "mem_cap_bytes": cfg.mem_cap_bytes, "guard_us": guard_ns / 1e3,
                   "gate_guard_us": (args.gate_guard_ns if args.gate_guard_ns else guard_ns) / 1e3 if args.device_gate else None},
        "gteps_in_kernel": edges / chunk_ns if chunk_ns else 0.0,
        "gteps_wall": edges / (wall_s * 1e9) if wall_s else 0.0,
        "bubble_fraction_of_epoch": bubble_ns / sum(r.epoch_ns for r, _ in with_task),
        "bubble_time_used": chunk_ns / bubble_ns if bubble_ns else 0.0,
        "bubble_breakdown": {"running": chunk_ns / bubble_ns, "insufficient_time": idle_ns / bubble_ns,
                             "runtime_and_guard": max(0.0, 1.0 - (chunk_ns + idle_ns) / bubble_ns), "no_memory": 0.0},
        # I = (T_with - T_no) / T_no (the paper's Section 6.1.5), against idle bubbles and against bubbles kept busy
        # without memory traffic; the same over the bursts' busy time only; and the bursts split by what precedes them
        "stage_slowdown_pct": pct(sa["epoch_ms_mean"], sb["epoch_ms_mean"]),
        "stage_slowdown_vs_busy_bubbles_pct": pct(sa["epoch_ms_mean"], sc["epoch_ms_mean"]),
        "stage_busy_slowdown_pct": pct(sa["busy_ms_mean"], sb["busy_ms_mean"]),
        "stage_busy_slowdown_vs_busy_bubbles_pct": pct(sa["busy_ms_mean"], sc["busy_ms_mean"]),
        "burst_slowdown_pct": {
            "first_after_bubble_vs_idle": pct(sa["burst_ms_first_after_bubble"], sb["burst_ms_first_after_bubble"]),
            "first_after_bubble_vs_busy": pct(sa["burst_ms_first_after_bubble"], sc["burst_ms_first_after_bubble"]),
            "others_vs_idle": pct(sa["burst_ms_others"], sb["burst_ms_others"]),
            "others_vs_busy": pct(sa["burst_ms_others"], sc["burst_ms_others"])},
        "arms": {"with_side_task": sa, "idle_bubbles": sb, "busy_bubbles_no_memory_traffic": sc,
                 "order": "B a A C a A B C (a: one untimed epoch with the side task)"},
        "steps_per_bubble": len(timed) / max(1, sum(r.n_bubbles for r, _ in with_task)),
        "mean_step_us": (chunk_ns / len(timed) / 1e3) if timed else None,
        "overruns": int(prog1.overruns - prog0.overruns), "deadline_misses": int(prog1.deadline_misses - prog0.deadline_misses),
        "runs_completed": int(prog1.runs_completed - prog0.runs_completed),
        "device_gate": args.device_gate, "steps_refused": int(prog1.steps_refused - prog0.steps_refused),
        "iterations_per_s_wall": (edges / E) / wall_s if wall_s else 0.0,
        "standalone_iteration_us": standalone_iter_ns / 1e3,
        "standalone_gbs": iter_bytes / standalone_iter_ns,
        "stage_tflops": ((fp_flops + bp_flops) * cfg.m / (sa["busy_ms_mean"] / 1e3) / 1e12) if fp_flops else None,
        "roofline": {"kernel": "k_scatter + k_gather (one PageRank iteration)", "bound": "hbm",
                     "achieved": pull_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": pull_gbs / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_note,
                     "traffic_gbs": traffic_gbs,
                     "traffic_frac_of_peak": (traffic_gbs / HBM_PEAK_GBS) if traffic_gbs else None,
                     "device_copy_gbs": copy_gbs,
                     "traffic_frac_of_device_copy": (traffic_gbs / copy_gbs) if traffic_gbs else None,
                     "iterations": iters_done,
                     "avg_iteration_us": (pull_ns / iters_done / 1e3) if iters_done else None,
                     "timing": "HIP events on the side stream around groups of %d steps, all inside the timed epochs" % ts,
                     "standalone_launch_us": {"k_scatter": s_ns / 1e3, "k_gather": g_ns / 1e3,
                                              "note": "whole sweeps outside bubbles, one event pair per launch"},
                     "in_bubble_over_standalone": in_bubble,
                     "launches": {"k_scatter": per_kind_n[1], "k_gather": per_kind_n[2], "k_finish": per_kind_n[3]},
                     "algorithmic_bytes_per_iteration": iter_bytes},
        "layout": {"messages_per_edge": info.messages / max(1, E), "ranges": info.ranges,
                   "merged_ranges": info.merged_ranges, "gather_tiles": info.gather_tiles,
                   "scatter_tiles": info.scatter_tiles, "gather_slots": info.gather_slots, "scatter_slots": info.scatter_slots,
                   "bytes_resident": info.bytes_resident, "bytes_peak_init": info.bytes_peak},
    }
    got = ranks.cpu().numpy()
    task.fr_pagerank_destroy(); stage.fr_stage_destroy(); load.fr_load_destroy(); ctx.fr_destroy()
    del rp, col, od, ranks, ws
    torch.cuda.empty_cache()

    # ---- the harvested ranks against the fp64 oracle (the run that is timed as the CPU baseline), element by element
    if not args.no_check:
        from oracle.pagerank import pagerank
        if out["runs_completed"] < 1:
            raise SystemExit("bench.py: %s completed no PageRank run inside the timed epochs; nothing to check" % cfg.name)
        tc = time.perf_counter()
        want, used = pagerank(g.row_ptr, g.col, g.out_degree, cfg.damping, K, n_threads=0, return_threads=True)
        dt = time.perf_counter() - tc
        err = np.abs(got.astype(np.float64) - want)
        big = want > 1.0 / V
        out["parity"] = {"max_abs_err": float(err.max()), "max_rel_err": float((err[big] / want[big]).max()) if big.any() else 0.0,
                         "sum_minus_one": float(got.astype(np.float64).sum() - 1.0),
                         "against": "fp64 CPU oracle, all %d vertices, %d iterations" % (V, K),
                         "tolerance_abs": PARITY_TOL_ABS, "tolerance_rel": PARITY_TOL_REL}
        log("%s parity: max abs %.3e, max rel %.3e (oracle %.1f s on %d threads)" % (cfg.name, out["parity"]["max_abs_err"], out["parity"]["max_rel_err"], dt, used))
        if out["parity"]["max_abs_err"] > PARITY_TOL_ABS or out["parity"]["max_rel_err"] > PARITY_TOL_REL:
            print(json.dumps(out))
            raise SystemExit("bench.py: %s ranks differ from the oracle beyond the tolerance" % cfg.name)
        out["cpu_baseline"] = {"value": K * E / dt / 1e9, "unit": "GTEPS", "cores": used, "kind": "oracle",
                               "sample": "%d iterations of the fp64 oracle on the same graph (%.1f s): the run the ranks are checked against" % (K, dt),
                               "cpu_model": cpu_model()}
        if headline and not args.no_cpu_baseline:
            # the fp32 row-parallel loop, one thread and all of them, on a bounded number of iterations
            from oracle.pagerank import pagerank_f32
            it1 = max(1, int((1 << 31) // max(1, E)))
            tc = time.perf_counter(); pagerank_f32(g.row_ptr, g.col, g.out_degree, cfg.damping, it1, n_threads=1); d1 = time.perf_counter() - tc
            itn = max(2, min(K, 8 * it1))
            tc = time.perf_counter(); _, usedn = pagerank_f32(g.row_ptr, g.col, g.out_degree, cfg.damping, itn, n_threads=0, return_threads=True); dn = time.perf_counter() - tc
            out["cpu_baseline"]["fp32_row_parallel"] = {
                "one_thread_gteps": it1 * E / d1 / 1e9, "one_thread_iterations_per_s": it1 / d1,
                "all_threads_gteps": itn * E / dn / 1e9, "all_threads_iterations_per_s": itn / dn, "threads": usedn,
                "sample": "%d iteration(s) on one thread (%.1f s), %d on %d threads (%.1f s), set-up included" % (it1, d1, itn, usedn, dn)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed epochs with the side task; 0 = 8 for cfg5 (2.5 s epochs), 12 otherwise")
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="cfg5")
    ap.add_argument("--per-config", type=int, default=1,
                    help="1: with the default configuration, also run cfg2, cfg3 and cfg4 (4 timed epochs each) and report them under per_config")
    ap.add_argument("--derate", type=float, default=1.25, help="first model = measured standalone cost x derate")
    ap.add_argument("--margin", type=float, default=1.02, help="final model = measured in-bubble step cost x margin")
    ap.add_argument("--guard-ns", type=int, default=0,
                    help="least time the host's plan keeps free at the end of every bubble; 0 = 60 us with the device gate (which "
                         "stops by the GPU's clock what the plan got wrong), 150 us without (covers the slow first sweeps after a burst)")
    ap.add_argument("--time-steps", type=int, default=16,
                    help="steps per HIP-event timing group in the measured epochs (an event between two kernels idles the GPU ~3 us)")
    ap.add_argument("--device-gate", type=int, default=1,
                    help="1 (default): the steps also check the GPU clock, when their kernel starts and before a workgroup takes another "
                         "tile, and stop where the bubble's time is up; what was not done is taken up in the next bubble.  "
                         "0: the host's plan alone (a little more bubble time used, and now and then a step that ends late)")
    ap.add_argument("--gate-guard-ns", type=int, default=50_000,
                    help="the device gate's own guard (its clock is the GPU's: it needs no allowance for the host model's drift over a bubble); 0 = --guard-ns")
    ap.add_argument("--adapt-costs", type=int, default=1,
                    help="1: the runtime's running profiler also scales the step costs by what the timed groups show (in the timed epochs; PageRank only: Graph SGD is harvested 2 percent better with its frozen model, 0 overruns either way)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the fp32 CPU loops (the fp64 oracle still runs, as the parity check)")
    ap.add_argument("--no-check", action="store_true", help="skip the oracle altogether (profiling runs): no parity, no cpu_baseline")
    ap.add_argument("--sgd-margin", type=float, default=1.08, help="--side-task sgd: final model = measured in-bubble step cost x this")
    ap.add_argument("--side-task", default="pagerank", choices=("pagerank", "sgd"),
                    help="sgd: the Graph SGD side task in the bubbles of cfg2's stage (a second line of its own, not the headline metric)")
    ap.add_argument("--interleave", type=int, default=0,
                    help="run the configuration's stage under interleaved 1F1B with this many model chunks (1F1B configurations): shorter bubbles, a second bubble workload")
    ap.add_argument("--profile-standalone", action="store_true",
                    help="stop after the standalone profile of the side task (for rocprofv3 counter runs: every sweep dispatch is a whole sweep)")
    ap.add_argument("--dump-events", default=None, help="write the timed epochs' event log (one JSON object per line) here")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py runs on one GPU only (--gpus 1).", file=sys.stderr)
        sys.exit(2)

    if args.side_task == "sgd":
        if not args.steps:
            args.steps = 12
        from bench_sgd import run as run_sgd
        return run_sgd(args, stage_load, log)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    steps = args.steps if args.steps else (8 if args.config == "cfg5" else 12)
    out = run_config(args.config, steps, args.warmup, args, headline=True)
    out["paper_context"] = {"bubble_rate_pct": 42.4, "cost_savings_pct": 7.8, "overhead_pct": 1.1,
                            "pagerank_iterations_per_s": 333.9, "hardware": "4x RTX 6000 Ada (paper, Section 6)"}
    if args.per_config and args.config == "cfg5":
        out["per_config"] = {}
        keep = ("value", "unit", "steps", "ms_per_step", "config", "gteps_in_kernel", "bubble_time_used", "stage_slowdown_pct",
                "stage_slowdown_vs_busy_bubbles_pct", "overruns", "deadline_misses", "device_gate", "steps_refused", "runs_completed",
                "standalone_iteration_us", "bubble_breakdown",
                "roofline", "layout", "parity", "cpu_baseline")
        for name in ("cfg2", "cfg3", "cfg4"):
            r = run_config(name, 4, 1, args, headline=False)
            out["per_config"][name] = {k: r[k] for k in keep if k in r}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
