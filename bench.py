#!/usr/bin/env python3
"""Benchmark of the bubble-harvesting hot path on one MI355X.

One step = one pipeline epoch of the emulated stage (its FP/BP GEMM bursts and the waits that stand for the
other stages) with the PageRank side task harvesting every bubble.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg2]
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
# HBM-side bytes one PageRank iteration (k_scatter + k_gather) moves on cfg2, from the FETCH_SIZE / WRITE_SIZE
# counter runs summarised under profiles/ (FETCH_SIZE scaled by 1.985, the factor a plain streaming kernel of known
# size shows).  Only valid for the kernels those counters were taken on: set to None when the kernels change.
CFG2_TRAFFIC_BYTES = 352.5e6


def log(*a):
    print(*a, file=sys.stderr, flush=True)


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=12)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--derate", type=float, default=1.25, help="first model = measured standalone cost x derate")
    ap.add_argument("--margin", type=float, default=1.02, help="final model = measured in-bubble step cost x margin")
    ap.add_argument("--guard-ns", type=int, default=150_000,
                    help="time kept free at the end of every bubble (covers the slow first sweeps after a burst)")
    ap.add_argument("--time-steps", type=int, default=16,
                    help="steps per HIP-event timing group in the measured epochs (an event between two kernels idles the GPU ~3 us)")
    ap.add_argument("--device-gate", type=int, default=0,
                    help="1: every step also checks the GPU clock when its kernel starts and does nothing if it would end late")
    ap.add_argument("--adapt-costs", type=int, default=1,
                    help="1: the runtime's running profiler also scales the step costs by what the timed groups show (in the timed epochs; PageRank only: Graph SGD is harvested 2 percent better with its frozen model, 0 overruns either way)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sgd-margin", type=float, default=1.08, help="--side-task sgd: final model = measured in-bubble step cost x this")
    ap.add_argument("--side-task", default="pagerank", choices=("pagerank", "sgd"),
                    help="sgd: the Graph SGD side task in the same stage's bubbles (a second line of its own, not the headline metric)")
    ap.add_argument("--dump-events", default=None, help="write the timed epochs' event log (one JSON object per line) here")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py runs on one GPU only (--gpus 1).", file=sys.stderr)
        sys.exit(2)

    if args.side_task == "sgd":
        from bench_sgd import run as run_sgd
        return run_sgd(args, stage_load, log)

    import numpy as np
    import torch

    import paper_2409_06941_amd as fr
    from workloads import configs

    cfg = configs.by_name(args.config)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    t_setup = time.time()
    g = cfg.build_graph()
    V, E, K = g.n_vertices, g.n_edges, cfg.iterations
    log("graph %s: V=%d E=%d built in %.1fs" % (cfg.name, V, E, time.time() - t_setup))
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    rp, col, od = dev(g.row_ptr), dev(g.col), dev(g.out_degree)
    ranks = torch.zeros(V, dtype=torch.float32, device="cuda")
    stage_stream = torch.cuda.Stream()

    load, ws, f_ns, b_ns, fp_flops, bp_flops = stage_load(cfg, stage_stream)
    log("stage load: f=%.3f ms b=%.3f ms" % (f_ns / 1e6, b_ns / 1e6))

    # ---- side-task profile: per-step costs from a few standalone iterations (the paper's side-task profiler)
    side_probe = fr.Context(device_id=0, cu_count=cfg.cu_count if cfg.cu_count < 256 else 0)
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
    log("layout: M/E=%.3f, %d ranges (%d with edges, %d merged), %d gather tiles, %d scatter tiles, init+first run %.2fs" %
        (info.messages / max(1, E), info.ranges, info.nonempty_ranges, info.merged_ranges, info.gather_tiles,
         info.scatter_tiles, t_init))
    log("standalone per iteration: scatter %.1f us, gather %.1f us (once per run: first vertex pass %.1f us, finish %.1f us)" %
        (s_ns / 1e3, g_ns / 1e3, v_ns / 1e3, h_ns / 1e3))
    log("shortest steps (one tile per launch): vertex %.1f us, scatter %.1f us, gather %.1f us, finish %.1f us" %
        tuple(x / 1e3 for x in one_tile_ns))
    standalone_iter_ns = s_ns + g_ns

    # ---- runtime, task, stage
    mem_cap = cfg.mem_cap_bytes if cfg.mem_cap_bytes else (64 << 30)
    kind = fr.FR_SCHED_1F1B if cfg.schedule == "1f1b" else fr.FR_SCHED_GPIPE
    stage = fr.Stage(kind, cfg.p, cfg.m, cfg.stage, f_ns, b_ns, load, stage_stream)
    n_segs = 2 * K + 2
    seg_kind = lambda g: (fr.FR_PR_SEG_VERTEX if g == 0 else fr.FR_PR_SEG_FINISH if g == n_segs - 1
                          else fr.FR_PR_SEG_SCATTER + ((g - 1) & 1))

    def start_task(launch_cost_ns, model, time_steps, adapt=0):
        ctx = fr.Context(device_id=0, cu_count=cfg.cu_count if cfg.cu_count < 256 else 0,
                         mem_available_bytes=mem_cap + 1, guard_ns=args.guard_ns, launch_cost_ns=launch_cost_ns,
                         max_chunk_ns=0, max_inflight=32, time_steps=time_steps, event_log_capacity=1 << 18,
                         device_gate=args.device_gate, adapt_costs=adapt)
        task = fr.PageRankTask(V, E, rp, col, od, ranks, damping=cfg.damping, iterations=K, max_runs=0,
                               mem_limit_bytes=mem_cap, **model)
        tid = ctx.fr_task_register(task.ops, task.user, task.profile)
        ctx.fr_bubble_begin(fr.fr_now_ns(), 5_000_000_000)          # a long first bubble for InitSideTask
        t_end = time.time() + 60
        while ctx.fr_query_progress(tid).state == fr.FR_CREATED and time.time() < t_end:
            time.sleep(0.001)
        ctx.fr_bubble_end()
        return ctx, task, tid

    # Second profiling pass, in place: an epoch (the fourth after the start) shows what a step costs inside real
    # bubbles, launch gaps included.  It is done twice: first with the standalone model, generously derated, then
    # with what the first pass measured - a bubble's first steps run some percent slower than its later ones, so a
    # pass that plans fewer steps per bubble than the timed epochs will measures a slower average than theirs.
    # The final model is the second pass's cost plus a small margin.
    ts = max(1, args.time_steps)
    standalone = (v_ns, s_ns, g_ns, h_ns)
    n_tiles = None
    def in_bubble_ratio(launch_cost_ns, model):
        nonlocal n_tiles
        ctx, task, tid = start_task(launch_cost_ns, model, ts)
        for _ in range(3):                       # untimed: right after a start the steps run a few percent slower
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
    if ratios:
        log("  group ratios min %.3f quartiles %.3f %.3f %.3f max %.3f" % ((min(ratios),) + tuple(statistics.quantiles(ratios, n=4)) + (max(ratios),)))
    one_tile_ns = [x * in_bubble for x in one_tile_standalone]
    ctx, task, tid = start_task(0, rates(*insitu, args.margin), ts, args.adapt_costs)     # the measured group times already hold the launch gaps
    def epochs(n, with_task):
        out = []
        for _ in range(n):
            out.append(stage.fr_stage_run_epoch(ctx if with_task else None))
        return out

    epochs(max(1, args.warmup), True)            # includes the bubble that initialises the task
    torch.cuda.synchronize()
    base_a = epochs((args.steps + 1) // 2, False)
    epochs(1, True)                              # untimed: the side task's first bubbles after a pause run ~6 % slower
    ctx.fr_event_log_clear()
    p0 = ctx.fr_query_progress(tid)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    with_task = epochs(args.steps, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    p1 = ctx.fr_query_progress(tid)
    base_b = epochs(args.steps // 2 if args.steps > 1 else 1, False)
    time.sleep(0.05)
    events = ctx.fr_event_log(1 << 18)
    p1 = ctx.fr_query_progress(tid)
    ctx.fr_task_stop(tid)

    if args.dump_events:
        with open(args.dump_events, "w") as fh:
            for r in with_task:
                fh.write(json.dumps({"epoch_ns": r.epoch_ns, "busy_ns": r.busy_ns, "bubble_ns": r.bubble_ns,
                                     "n_bubbles": r.n_bubbles, "overruns": r.overruns}) + "\n")
            for e in events:
                fh.write(json.dumps({"kind": e.kind, "bubble": e.bubble, "run": e.run, "segment": e.segment,
                                     "tile0": e.tile0, "tile1": e.tile1, "modelled_ns": e.modelled_ns,
                                     "measured_ns": e.measured_ns, "t_host_ns": e.t_host_ns}) + "\n")
    wall_s = t1 - t0
    edges = p1.work_units_done - p0.work_units_done
    bubble_ns = sum(r.bubble_ns for r in with_task)
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
    per_kind_n = [sum(1 for e in timed if seg_kind(e.segment) == k) for k in range(4)]
    timed_edges = sum(e.work_units for e in timed)
    # One iteration = one scatter + one gather launch and moves 4E + 24V + 4 algorithmic bytes (col entries, row starts, one
    # compulsory read of every contribution, the rank write, and the vertex pass); iterations done = edges / E.
    iters_done = timed_edges / E
    pull_ns = sum(e.measured_ns for e in timed)
    pull_bytes = iters_done * (4.0 * E + 24.0 * V + 4.0)
    pull_gbs = pull_bytes / pull_ns if pull_ns else 0.0
    iter_bytes = 4.0 * E + 24.0 * V + 4.0
    e_with = statistics.mean(r.epoch_ns for r in with_task)
    base = base_a + base_b
    e_without = statistics.mean(r.epoch_ns for r in base)
    ew, eo = [r.epoch_ns for r in with_task], [r.epoch_ns for r in base]
    busy_with = statistics.mean(r.busy_ns for r in with_task)
    busy_without = statistics.mean(r.busy_ns for r in base)

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

    out = {
        "metric": "side-task GTEPS harvested in bubbles",
        "value": edges / bubble_ns if bubble_ns else 0.0,
        "unit": "GTEPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_s * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %s p=%d m=%d stage=%d; PageRank on %s 2^%d vertices, %d edges, %d iterations, seed %d"
                   % (cfg.name, cfg.schedule, cfg.p, cfg.m, cfg.stage, cfg.graph, cfg.scale, E, K, cfg.seed),
                   "stage_load": ("bf16 GEMM bursts: %d GPT layers h=%d ffn=%d tokens=%d" %
                                  (cfg.load.layers, cfg.load.hidden, cfg.load.ffn, cfg.load.tokens)) if cfg.load else "busy-wait",
                   "f_ms": f_ns / 1e6, "b_ms": b_ns / 1e6, "cu_count": cfg.cu_count},
        "gteps_in_kernel": edges / chunk_ns if chunk_ns else 0.0,
        "gteps_wall": edges / (wall_s * 1e9),
        "bubble_fraction_of_epoch": bubble_ns / sum(r.epoch_ns for r in with_task),
        "bubble_time_used": chunk_ns / bubble_ns if bubble_ns else 0.0,
        "bubble_breakdown": {"running": chunk_ns / bubble_ns, "insufficient_time": idle_ns / bubble_ns,
                             "runtime_and_guard": max(0.0, 1.0 - (chunk_ns + idle_ns) / bubble_ns), "no_memory": 0.0},
        "stage_slowdown_pct": 100.0 * (e_with - e_without) / e_without,
        "stage_busy_slowdown_pct": 100.0 * (busy_with - busy_without) / busy_without,
        "epoch_ms_with": e_with / 1e6, "epoch_ms_without": e_without / 1e6,
        "epoch_ms_with_min_med_max": [min(ew) / 1e6, statistics.median(ew) / 1e6, max(ew) / 1e6],
        "epoch_ms_without_min_med_max": [min(eo) / 1e6, statistics.median(eo) / 1e6, max(eo) / 1e6],
        "stage_slowdown_pct_of_medians": 100.0 * (statistics.median(ew) - statistics.median(eo)) / statistics.median(eo),
        "steps_per_bubble": len(timed) / max(1, sum(r.n_bubbles for r in with_task)),
        "mean_step_us": (chunk_ns / len(timed) / 1e3) if timed else None,
        "overruns": int(p1.overruns - p0.overruns), "deadline_misses": int(p1.deadline_misses - p0.deadline_misses),
        "runs_completed": int(p1.runs_completed - p0.runs_completed),
        "device_gate": args.device_gate, "steps_refused": int(p1.steps_refused - p0.steps_refused),
        "iterations_per_s_wall": (edges / E) / wall_s,
        "standalone_iteration_us": standalone_iter_ns / 1e3,
        "standalone_gbs": iter_bytes / standalone_iter_ns,
        "stage_tflops": ((fp_flops + bp_flops) * cfg.m / (busy_with / 1e9) / 1e12) if fp_flops else None,
        "roofline": {"kernel": "k_scatter + k_gather (one PageRank iteration)", "bound": "hbm",
                     "achieved": pull_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": pull_gbs / HBM_PEAK_GBS,
                     "traffic": CFG2_TRAFFIC_BYTES if cfg.name == "cfg2" else None,
                     "traffic_gbs": (CFG2_TRAFFIC_BYTES * iters_done / pull_ns) if (cfg.name == "cfg2" and pull_ns) else None,
                     "traffic_frac_of_peak": (CFG2_TRAFFIC_BYTES * iters_done / pull_ns / HBM_PEAK_GBS) if (cfg.name == "cfg2" and pull_ns) else None,
                     "device_copy_gbs": copy_gbs,
                     "traffic_frac_of_device_copy": (CFG2_TRAFFIC_BYTES * iters_done / pull_ns / copy_gbs) if (cfg.name == "cfg2" and pull_ns) else None,
                     "iterations": iters_done,
                     "avg_iteration_us": (pull_ns / iters_done / 1e3) if iters_done else None,
                     "timing": "HIP events on the side stream around groups of %d steps, all inside the timed epochs" % max(1, args.time_steps),
                     "standalone_launch_us": {"k_scatter": s_ns / 1e3, "k_gather": g_ns / 1e3,
                                              "note": "whole sweeps outside bubbles, one event pair per launch"},
                     "in_bubble_over_standalone": in_bubble,
                     "launches": {"k_scatter": per_kind_n[1], "k_gather": per_kind_n[2], "k_finish": per_kind_n[3]},
                     "algorithmic_bytes_per_iteration": 4.0 * E + 24.0 * V + 4.0},
        "layout": {"messages_per_edge": info.messages / max(1, E), "ranges": info.ranges,
                   "merged_ranges": info.merged_ranges, "gather_tiles": info.gather_tiles,
                   "scatter_tiles": info.scatter_tiles,
                   "bytes_resident": info.bytes_resident, "bytes_peak_init": info.bytes_peak},
        "paper_context": {"bubble_rate_pct": 42.4, "cost_savings_pct": 7.8, "overhead_pct": 1.1,
                          "pagerank_iterations_per_s": 333.9, "hardware": "4x RTX 6000 Ada (paper, Section 6)"},
    }

    if not args.no_cpu_baseline:
        from oracle.pagerank import pagerank
        cpu_iters = 600
        tc = time.perf_counter()
        _, used = pagerank(g.row_ptr, g.col, g.out_degree, cfg.damping, cpu_iters, n_threads=0, return_threads=True)
        dt = time.perf_counter() - tc
        out["cpu_baseline"] = {"value": cpu_iters * E / dt / 1e9, "unit": "GTEPS", "cores": used, "kind": "oracle",
                               "sample": "%d iterations of the fp64 oracle on the same graph (%.1f s)" % (cpu_iters, dt)}
    task.fr_pagerank_destroy(); stage.fr_stage_destroy(); load.fr_load_destroy(); ctx.fr_destroy()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
