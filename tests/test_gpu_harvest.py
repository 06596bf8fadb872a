"""GPU: PageRank harvested inside the bubbles of an emulated stage, against the oracle's plan and the oracle's ranks."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2409_06941_amd as fr          # noqa: E402
from oracle import planner, schedule       # noqa: E402
from oracle.pagerank import pagerank       # noqa: E402
from workloads import configs, graphs      # noqa: E402

NAMES = {fr.FR_EV_INIT: "INIT", fr.FR_EV_CHUNK: "CHUNK", fr.FR_EV_IDLE: "IDLE", fr.FR_EV_MISS: "MISS", fr.FR_EV_OVERRUN: "OVERRUN"}


def _dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).cuda()


def _init_bubble(ctx, tid, length_ns=2_000_000_000):
    """One long bubble for InitSideTask (Algorithm 2: the first bubble that finds the task CREATED initialises it)."""
    import time
    ctx.fr_bubble_begin(fr.fr_now_ns(), length_ns)
    deadline = time.time() + 30
    while ctx.fr_query_progress(tid).state == fr.FR_CREATED and time.time() < deadline:
        time.sleep(0.001)
    return ctx.fr_bubble_end()


def _segments(task, iterations):
    v = task.fr_pagerank_tile_costs(fr.FR_PR_SEG_VERTEX)
    s = task.fr_pagerank_tile_costs(fr.FR_PR_SEG_SCATTER)
    g = task.fr_pagerank_tile_costs(fr.FR_PR_SEG_GATHER)
    h = task.fr_pagerank_tile_costs(fr.FR_PR_SEG_FINISH)
    segs = [v]
    for _ in range(iterations):
        segs += [s, g]
    return segs + [h]


def _scaled_model(share, phase_ns, iterations, gather_weight, scatter_weight, info):
    """Rates that make the task's cost model claim `share` of the measured time of every sweep."""
    V0_rows = info.ranges * info.rows_per_partition
    pv = max(1, int(share * phase_ns[0] * 1e6 / V0_rows))
    s_fs = share * phase_ns[1] / iterations * 1e6
    g_fs = share * phase_ns[2] / iterations * 1e6
    pm = max(1, int(s_fs / max(1, info.messages + scatter_weight)))
    pe = max(1, int(2 * g_fs / max(1, gather_weight)))
    return dict(fs_per_vertex=pv, fs_per_message=pm, fs_per_edge=pe, finish_tile_ns=1000)


def _floors(min_step_ns, iterations):
    fv, fs, fg, fh = min_step_ns
    return [fv] + [fs, fg] * iterations + [fh]


def _check_cost_rule(task, pe, pm, pv, hub_ns):
    """Tile costs follow the documented integer formula."""
    rows = task.fr_pagerank_tile_work(fr.FR_PR_SEG_VERTEX)
    assert task.fr_pagerank_tile_costs(fr.FR_PR_SEG_VERTEX) == [max(1, -(-r * pv // 10**6)) for r in rows]
    info = task.fr_pagerank_info()
    edges = task.fr_pagerank_tile_work(fr.FR_PR_SEG_GATHER)
    R = info.rows_per_partition
    weights = task.fr_pagerank_tile_weights(fr.FR_PR_SEG_GATHER)
    assert all(w >= 2 * e + 147456 for w, e in zip(weights, edges))     # 2 edges + 6 repeated edges + 147456 a piece
    assert task.fr_pagerank_tile_costs(fr.FR_PR_SEG_GATHER) == [max(1, -(-(w * pe // 2) // 10**6)) for w in weights]
    msgs = task.fr_pagerank_tile_work(fr.FR_PR_SEG_SCATTER)
    srcs = task.fr_pagerank_tile_weights(fr.FR_PR_SEG_SCATTER)
    assert task.fr_pagerank_tile_costs(fr.FR_PR_SEG_SCATTER) == [max(1, -(-((m + s) * pm) // 10**6)) for m, s in zip(msgs, srcs)]
    assert len(edges) == info.gather_tiles
    empty = info.ranges - info.nonempty_ranges
    assert task.fr_pagerank_tile_costs(fr.FR_PR_SEG_FINISH) == [hub_ns] * max(1, (info.merged_ranges + empty) * (R // 2048))


def test_config1_harvest_matches_plan_and_oracle_bits():
    cfg = configs.by_name("cfg1")
    g = cfg.build_graph()
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    ref = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")

    # reference bits: one unchunked run outside any bubble
    t_ref = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ref, iterations=cfg.iterations)
    t_ref.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    t_ref.fr_pagerank_destroy()

    guard, launch, max_chunk = 300_000, 25_000, 500_000
    # shortest-step floors (vertex, scatter, gather, finish): above one tile's cost for scatter and gather, so
    # that steps of a tile or two are charged the floor and longer steps the sum
    floors = (9_000, 60_000, 80_000, 20_000)
    ctx = fr.Context(device_id=0, guard_ns=guard, launch_cost_ns=launch, max_chunk_ns=max_chunk, time_steps=1,
                     mem_available_bytes=1 << 40)
    task = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=cfg.iterations, max_runs=3,
                           mem_limit_bytes=1 << 30, fs_per_edge=260_000, fs_per_message=400_000, fs_per_vertex=300_000,
                           finish_tile_ns=15000, min_step_ns=floors)
    tid = ctx.fr_task_register(task.ops, task.user, task.profile)
    assert _init_bubble(ctx, tid) == fr.FR_OK
    assert ctx.fr_query_progress(tid).state == fr.FR_PAUSED
    stream = torch.cuda.Stream()
    load = fr.Load(fr.FR_LOAD_BUSYWAIT, fp_ns=cfg.busy_fp_ns, bp_ns=cfg.busy_bp_ns)
    stage = fr.Stage(fr.FR_SCHED_1F1B, cfg.p, cfg.m, cfg.stage, cfg.busy_fp_ns, cfg.busy_bp_ns, load, stream)
    n_epochs = 3
    results = []
    for ep in range(n_epochs):
        print("epoch", ep, flush=True)
        results.append(stage.fr_stage_run_epoch(ctx))
    pr = ctx.fr_query_progress(tid)
    log = ctx.fr_event_log()
    segs = _segments(task, cfg.iterations)          # the cost tables exist once InitSideTask has run
    info = task.fr_pagerank_info()
    _check_cost_rule(task, 260_000, 400_000, 300_000, 15000)
    ctx.fr_task_stop(tid)
    got = ranks.cpu().numpy()
    want_bits = ref.cpu().numpy()
    task.fr_pagerank_destroy()
    stage.fr_stage_destroy()
    load.fr_load_destroy()
    ctx.fr_destroy()

    windows, T = schedule.bubbles("1f1b", cfg.p, cfg.m, cfg.busy_fp_ns, cfg.busy_bp_ns, cfg.stage)
    lengths = [2_000_000_000] + [e - a for a, e in windows] * n_epochs
    assert [r.n_bubbles for r in results] == [len(windows)] * n_epochs
    assert pr.overruns == 0 and pr.deadline_misses == 0 and sum(r.overruns for r in results) == 0
    assert pr.bubbles_seen == len(lengths)

    slots = [0] + [info.scatter_slots, info.gather_slots] * cfg.iterations + [0]
    want = planner.plan(lengths, segs, guard, launch, max_chunk, max_runs=3, floors=_floors(floors, cfg.iterations), slots=slots)
    # (the rules of the step cost - floor, sum, steps of up to a round - are pinned on the planner by the CPU tests;
    # here the log must follow whatever the plan says)
    got_log = [(NAMES[e.kind], e.bubble, e.run, e.segment, e.tile0, e.tile1, e.modelled_ns) for e in log]
    want_log = [(r.kind, r.bubble, r.run, r.segment, r.tile0, r.tile1, r.modelled_ns) for r in want]
    assert got_log == want_log
    # edges accounted exactly: every completed run traverses K * E edges
    edges = sum(e.work_units for e in log if e.kind == fr.FR_EV_CHUNK)
    assert pr.runs_completed == 3 and edges == 3 * cfg.iterations * g.n_edges == pr.work_units_done
    # every chunk got a measured GPU time
    assert all(e.measured_ns > 0 for e in log if e.kind == fr.FR_EV_CHUNK)

    assert np.array_equal(got.view(np.uint32), want_bits.view(np.uint32))       # chunked == unchunked, bit for bit
    oracle = pagerank(g.row_ptr, g.col, g.out_degree, cfg.damping, cfg.iterations)
    assert np.abs(got.astype(np.float64) - oracle).max() <= 1e-5
    # the stage's epoch is the ideal schedule plus measured op stretch; it cannot be shorter than the ideal
    assert all(r.epoch_ns >= T for r in results)


def test_harvest_in_rounds_matches_plan_and_oracle():
    # On a stream of 8 CUs a launch has 16 workgroups, and this uniform graph of 16.8 M edges is cut into hundreds of
    # tiles per sweep, which the workgroups hand out among themselves.  Steps that end inside a sweep are cut to
    # whole rounds of 16 tiles: the runtime's log is the plan of the oracle's planner with that rule, record for
    # record, and the ranks are the standalone run's bits and the fp64 oracle's values.
    K = 3
    g = graphs.fixed_outdeg_csr(1 << 20, 16, seed=34)
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    ref = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    guard, launch, max_chunk = 300_000, 10_000, 10**12
    floors = (20_000, 150_000, 150_000, 20_000)
    ctx = fr.Context(device_id=0, cu_count=8, guard_ns=guard, launch_cost_ns=launch, max_chunk_ns=max_chunk, time_steps=1,
                     mem_available_bytes=1 << 40)
    t_ref = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ref, iterations=K)
    t_ref.fr_pagerank_run_standalone(0, ctx.fr_side_stream())         # same CU mask, hence the same layout
    t_ref.fr_pagerank_destroy()
    # a cost model well above what the sweeps take on 8 CUs (about 1.6 ms each), so that nothing overruns
    task = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=K, max_runs=1, mem_limit_bytes=1 << 32,
                           fs_per_edge=400_000, fs_per_message=400_000, fs_per_vertex=100_000, finish_tile_ns=5_000,
                           min_step_ns=floors)
    tid = ctx.fr_task_register(task.ops, task.user, task.profile)
    assert _init_bubble(ctx, tid) == fr.FR_OK
    stream = torch.cuda.Stream()
    f_ns, b_ns = 3_000_000, 6_000_000
    load = fr.Load(fr.FR_LOAD_BUSYWAIT, fp_ns=f_ns, bp_ns=b_ns)
    stage = fr.Stage(fr.FR_SCHED_1F1B, 4, 8, 2, f_ns, b_ns, load, stream)
    results = []
    for ep in range(6):
        print("epoch", ep, flush=True)
        results.append(stage.fr_stage_run_epoch(ctx))
        if ctx.fr_query_progress(tid).runs_completed >= 1:
            break
    pr = ctx.fr_query_progress(tid)
    log = ctx.fr_event_log()
    segs = _segments(task, K)
    info = task.fr_pagerank_info()
    ctx.fr_task_stop(tid)
    got, want_bits = ranks.cpu().numpy(), ref.cpu().numpy()
    task.fr_pagerank_destroy(); stage.fr_stage_destroy(); load.fr_load_destroy(); ctx.fr_destroy()

    assert info.scatter_slots == 16 and info.gather_slots == 16       # two workgroups per CU at these sizes
    assert len(segs[1]) >= 4 * info.scatter_slots and len(segs[2]) >= 4 * info.gather_slots
    assert pr.runs_completed == 1 and pr.overruns == 0 and pr.deadline_misses == 0
    windows, _ = schedule.bubbles("1f1b", 4, 8, f_ns, b_ns, 2)
    lengths = [2_000_000_000] + [e - a for a, e in windows] * len(results)
    slots = [0] + [info.scatter_slots, info.gather_slots] * K + [0]
    want = planner.plan(lengths, segs, guard, launch, max_chunk, max_runs=1, floors=_floors(floors, K), slots=slots)
    got_log = [(NAMES[e.kind], e.bubble, e.run, e.segment, e.tile0, e.tile1, e.modelled_ns) for e in log]
    want_log = [(r.kind, r.bubble, r.run, r.segment, r.tile0, r.tile1, r.modelled_ns) for r in want]
    assert got_log == want_log[:len(got_log)] and len(got_log) >= len([r for r in want if r.kind == "CHUNK"])
    cut = [r for r in want if r.kind == "CHUNK" and slots[r.segment] and r.tile1 - r.tile0 > slots[r.segment] and r.tile1 < len(segs[r.segment])]
    assert cut and all((r.tile1 - r.tile0) % slots[r.segment] == 0 for r in cut)      # the rule was at work
    assert sum(e.work_units for e in log if e.kind == fr.FR_EV_CHUNK) == K * g.n_edges
    assert np.array_equal(got.view(np.uint32), want_bits.view(np.uint32))
    oracle = pagerank(g.row_ptr, g.col, g.out_degree, 0.85, K)
    assert np.abs(got.astype(np.float64) - oracle).max() <= 1e-5
    big = oracle > 1.0 / g.n_vertices
    assert (np.abs(got[big] - oracle[big]) / oracle[big]).max() <= 1e-4


def test_harvest_in_the_bubbles_of_an_interleaved_schedule_matches_plan_and_oracle():
    # Interleaved 1F1B with two model chunks per stage (bubble-reducing prior work, Sections 1 and 2.2.2): the same
    # stage idles half as long, in more and shorter windows.  The side task still lands in them exactly as the
    # oracle's planner says, and ends with the standalone run's bits and the oracle's values.
    cfg = configs.by_name("cfg1")
    g = cfg.build_graph()
    K = 10
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    ref = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    t_ref = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ref, iterations=K)
    t_ref.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    t_ref.fr_pagerank_destroy()
    guard, launch, max_chunk = 200_000, 25_000, 400_000
    floors = (9_000, 60_000, 80_000, 20_000)
    ctx = fr.Context(device_id=0, guard_ns=guard, launch_cost_ns=launch, max_chunk_ns=max_chunk, time_steps=1)
    task = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=K, max_runs=2,
                           fs_per_edge=260_000, fs_per_message=400_000, fs_per_vertex=300_000, finish_tile_ns=15000,
                           min_step_ns=floors)
    tid = ctx.fr_task_register(task.ops, task.user, task.profile)
    assert _init_bubble(ctx, tid) == fr.FR_OK
    p, m, v, s, f_ns, b_ns = 4, 8, 2, 2, 1_000_000, 2_000_000          # per chunk: half of cfg1's 2 ms / 4 ms
    stream = torch.cuda.Stream()
    load = fr.Load(fr.FR_LOAD_BUSYWAIT, fp_ns=v * f_ns, bp_ns=v * b_ns)     # a chunk's operation is 1 / v of the burst
    stage = fr.Stage(fr.FR_SCHED_INTERLEAVED, p, m, s, f_ns, b_ns, load, stream, chunks=v)
    n_epochs = 4
    results = [stage.fr_stage_run_epoch(ctx) for _ in range(n_epochs)]
    pr = ctx.fr_query_progress(tid)
    log = ctx.fr_event_log()
    info = task.fr_pagerank_info()
    segs = _segments(task, K)
    ctx.fr_task_stop(tid)
    got = ranks.cpu().numpy()
    task.fr_pagerank_destroy(); stage.fr_stage_destroy(); load.fr_load_destroy(); ctx.fr_destroy()

    windows, T = schedule.bubbles_interleaved(p, m, v, f_ns, b_ns, s)
    plain, T_plain = schedule.bubbles("1f1b", p, m, v * f_ns, v * b_ns, s)
    assert sum(e - a for a, e in windows) * v == sum(e - a for a, e in plain) and len(windows) > len(plain)
    assert [r.n_bubbles for r in results] == [len(windows)] * n_epochs
    assert [r.bubble_ns for r in results] == [sum(e - a for a, e in windows)] * n_epochs
    assert pr.overruns == 0 and pr.deadline_misses == 0
    lengths = [2_000_000_000] + [e - a for a, e in windows] * n_epochs
    slots = [0] + [info.scatter_slots, info.gather_slots] * K + [0]
    want = planner.plan(lengths, segs, guard, launch, max_chunk, max_runs=2, floors=_floors(floors, K), slots=slots)
    got_log = [(NAMES[e.kind], e.bubble, e.run, e.segment, e.tile0, e.tile1, e.modelled_ns) for e in log]
    want_log = [(r.kind, r.bubble, r.run, r.segment, r.tile0, r.tile1, r.modelled_ns) for r in want]
    assert got_log == want_log
    assert pr.runs_completed == 2
    assert np.array_equal(got.view(np.uint32), ref.cpu().numpy().view(np.uint32))
    _oracle_check(got, g, K)


def test_pagerank_task_is_stopped_alone_when_it_exceeds_its_memory_limit():
    g = graphs.rmat_csr(12, 1 << 15, seed=2)
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    ctx = fr.Context(device_id=0, mem_available_bytes=1 << 40)
    task = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=2, mem_limit_bytes=200_000)
    tid = ctx.fr_task_register(task.ops, task.user, task.profile)
    ctx.fr_bubble_begin(fr.fr_now_ns(), 50_000_000)
    import time
    time.sleep(0.05)
    assert ctx.fr_bubble_end() == fr.FR_OK
    pr = ctx.fr_query_progress(tid)
    assert pr.state == fr.FR_STOPPED and pr.last_error == fr.FR_ERR_OOM
    task.fr_pagerank_destroy()
    ctx.fr_destroy()


def test_admission_rejects_task_larger_than_the_bubbles_free_memory():
    g = graphs.rmat_csr(10, 3000, seed=2)
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    ctx = fr.Context(device_id=0, mem_available_bytes=1 << 20)
    task = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=2, mem_limit_bytes=1 << 20)
    with pytest.raises(fr.FreeRideError) as e:
        ctx.fr_task_register(task.ops, task.user, task.profile)
    assert e.value.code == fr.FR_ERR_NOMEM
    task.fr_pagerank_destroy()
    ctx.fr_destroy()


def test_cu_masked_side_stream_runs_the_same_bits():
    g = graphs.rmat_csr(14, 1 << 18, seed=0)
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    outs = []
    for cu in (0, 64):
        ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
        ctx = fr.Context(device_id=0, cu_count=cu)
        task = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=5)
        task.fr_pagerank_run_standalone(0, ctx.fr_side_stream())
        task.fr_pagerank_destroy()
        ctx.fr_destroy()
        outs.append(ranks.cpu().numpy())
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))


@pytest.mark.parametrize("grace_ns,killed", [(200_000, True), (0, False)])
def test_framework_enforced_limit_stops_a_task_whose_gpu_work_outlives_the_grace_period(grace_ns, killed):
    # a cost model that claims every step is free makes the worker enqueue up to max_inflight whole sweeps at the
    # very end of the bubble: about 2 ms of GPU work behind a 0.5 ms bubble (Section 4.5, framework-enforced limit)
    import time
    g = graphs.rmat_csr(22, 1 << 26, seed=1)
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    ctx = fr.Context(device_id=0, guard_ns=0, launch_cost_ns=0, time_steps=1, max_inflight=32, grace_ns=grace_ns)
    task = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=50, max_runs=0,
                           fs_per_edge=1, fs_per_message=1, fs_per_vertex=1, finish_tile_ns=1)
    tid = ctx.fr_task_register(task.ops, task.user, task.profile)
    assert _init_bubble(ctx, tid) == fr.FR_OK
    ctx.fr_bubble_begin(fr.fr_now_ns(), 500_000)
    time.sleep(0.0005)
    assert ctx.fr_bubble_end() == fr.FR_ERR_OVERRUN
    time.sleep(0.0004)                                   # past the grace period, the sweeps are still running
    ctx.fr_bubble_begin(fr.fr_now_ns(), 1_000)           # the verdict falls at the next bubble notification
    ctx.fr_bubble_end()
    time.sleep(0.05)
    pr = ctx.fr_query_progress(tid)
    if killed:
        assert pr.state == fr.FR_STOPPED and pr.last_error == fr.FR_ERR_OVERRUN and pr.killed == 1
        assert pr.mem_used_bytes > 0                     # what it held when it was stopped; released since
    else:
        assert pr.state == fr.FR_PAUSED and pr.killed == 0 and pr.overruns >= 1
        ctx.fr_task_stop(tid)
    task.fr_pagerank_destroy()
    ctx.fr_destroy()


def test_running_profiler_repairs_a_cost_model_that_claims_steps_are_much_cheaper_than_they_are():
    # The task's own model is set to 20 % of the measured step times.  With the frozen model the steps planned for
    # the end of a bubble run past it again and again; with adapt_costs the measured / modelled ratio of the first
    # steps scales the model up and the later epochs see no overrun.  The ranks keep the standalone run's bits.
    g = graphs.rmat_csr(21, 1 << 25, seed=9)
    V, E, K = g.n_vertices, g.n_edges, 20
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ref = torch.zeros(V, dtype=torch.float32, device="cuda")
    probe = fr.PageRankTask(V, E, rp, col, od, ref, iterations=K)
    probe.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    ph = probe.fr_pagerank_run_standalone(0, torch.cuda.current_stream(), want_phase_ns=True)
    info = probe.fr_pagerank_info()
    gw, sw = (sum(probe.fr_pagerank_tile_weights(k)) for k in (fr.FR_PR_SEG_GATHER, fr.FR_PR_SEG_SCATTER))
    probe.fr_pagerank_destroy()
    low = 0.2
    model = _scaled_model(low, ph, K, gw, sw, info)
    stream = torch.cuda.Stream()
    f_ns, b_ns = 1_000_000, 2_000_000
    load = fr.Load(fr.FR_LOAD_BUSYWAIT, fp_ns=f_ns, bp_ns=b_ns)
    late = {}
    for adapt in (0, 1):
        ranks = torch.zeros(V, dtype=torch.float32, device="cuda")
        ctx = fr.Context(device_id=0, guard_ns=20_000, launch_cost_ns=5_000, time_steps=1, adapt_costs=adapt)
        task = fr.PageRankTask(V, E, rp, col, od, ranks, iterations=K, max_runs=0, **model)
        tid = ctx.fr_task_register(task.ops, task.user, task.profile)
        assert _init_bubble(ctx, tid) == fr.FR_OK
        stage = fr.Stage(fr.FR_SCHED_1F1B, 4, 8, 2, f_ns, b_ns, load, stream)
        stage.fr_stage_run_epoch(ctx)                    # the running profiler learns here
        late[adapt] = sum(stage.fr_stage_run_epoch(ctx).overruns for _ in range(3))
        scales = ctx.fr_cost_scales()
        pr = ctx.fr_query_progress(tid)
        ctx.fr_task_stop(tid)
        got = ranks.cpu().numpy()
        task.fr_pagerank_destroy(); stage.fr_stage_destroy(); ctx.fr_destroy()
        print("adapt", adapt, "overruns in epochs 2-4:", late[adapt], "scales", scales[:4], "runs", pr.runs_completed, flush=True)
        assert pr.runs_completed >= 1
        assert np.array_equal(got.view(np.uint32), ref.cpu().numpy().view(np.uint32))
        _oracle_check(got, g, K)
        if adapt:
            assert all(s >= 2_500_000 for s in scales[1:3]), scales      # scatter and gather: about 1 / 0.2, or above
        else:
            assert scales == [1_000_000] * 8
    load.fr_load_destroy()
    assert late[0] > 0 and late[1] == 0, late


def test_running_profiler_changes_the_scales_between_bubbles_and_inside_one_only_after_a_step_that_is_far_off():
    # The model claims the standalone sweep times; every step is timed on its own.  The scales move when a bubble's
    # steps have been summed, before the next bubble is planned, and inside a bubble only after a step that took over
    # 1.25 times its scaled cost: in a bubble without such a step the logged cost of a whole gather sweep (scaled
    # cost + launch cost) is one number, and over the bubbles it takes several values.
    import time
    g = graphs.rmat_csr(21, 1 << 25, seed=9)
    V, E, K = g.n_vertices, g.n_edges, 20
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(V, dtype=torch.float32, device="cuda")
    probe = fr.PageRankTask(V, E, rp, col, od, ranks, iterations=K)
    probe.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    ph = probe.fr_pagerank_run_standalone(0, torch.cuda.current_stream(), want_phase_ns=True)
    info = probe.fr_pagerank_info()
    gw, sw = (sum(probe.fr_pagerank_tile_weights(k)) for k in (fr.FR_PR_SEG_GATHER, fr.FR_PR_SEG_SCATTER))
    probe.fr_pagerank_destroy()
    model = _scaled_model(1.0, ph, K, gw, sw, info)
    stream = torch.cuda.Stream()
    f_ns, b_ns = 1_000_000, 2_000_000
    load = fr.Load(fr.FR_LOAD_BUSYWAIT, fp_ns=f_ns, bp_ns=b_ns)
    launch_ns = 5_000
    ctx = fr.Context(device_id=0, guard_ns=100_000, launch_cost_ns=launch_ns, time_steps=1, adapt_costs=1, event_log_capacity=1 << 16)
    task = fr.PageRankTask(V, E, rp, col, od, ranks, iterations=K, max_runs=0, **model)
    tid = ctx.fr_task_register(task.ops, task.user, task.profile)
    assert _init_bubble(ctx, tid) == fr.FR_OK
    stage = fr.Stage(fr.FR_SCHED_1F1B, 4, 8, 2, f_ns, b_ns, load, stream)
    for _ in range(6):
        stage.fr_stage_run_epoch(ctx)
    time.sleep(0.05)
    scales = ctx.fr_cost_scales()
    events = ctx.fr_event_log(1 << 16)
    ctx.fr_task_stop(tid)
    task.fr_pagerank_destroy(); stage.fr_stage_destroy(); load.fr_load_destroy(); ctx.fr_destroy()
    sweeps, far_off = {}, set()      # bubble -> logged costs of its whole gather sweeps; bubbles with a step far off
    for e in events:
        if e.kind != fr.FR_EV_CHUNK:
            continue
        if e.measured_ns * 4 > (e.modelled_ns - launch_ns) * 5 * 0.97:       # (a little wider than the runtime's test)
            far_off.add(e.bubble)
        if e.tile0 == 0 and e.tile1 == info.gather_tiles and e.segment >= 2 and e.segment % 2 == 0:
            sweeps.setdefault(e.bubble, []).append(e.modelled_ns)
    quiet = [b for b in sweeps if b not in far_off and len(sweeps[b]) >= 2]
    print("scales", scales[:4], "bubbles with gather sweeps", len(sweeps), "without a step far off", len(quiet),
          "costs of a gather sweep", sorted({v[0] for v in sweeps.values()})[:6], flush=True)
    assert len(sweeps) >= 12, len(sweeps)       # (how many of them are without a step far off depends on the machine's hiccups)
    assert all(len(set(sweeps[b])) == 1 for b in quiet), {b: sorted(set(sweeps[b])) for b in quiet if len(set(sweeps[b])) > 1}
    assert len({sweeps[b][0] for b in sweeps}) >= 2
    assert scales[1] != 1_000_000 and scales[2] != 1_000_000


def _gate_accounts(log, pr):
    """What the device gate took back is consistent: every FR_EV_REFUSED record is a whole step of the log, or the tail
    of a step whose CHUNK record was shortened to the tiles it did; the progress counters hold what was done."""
    chunks = [e for e in log if e.kind == fr.FR_EV_CHUNK]
    refused = [e for e in log if e.kind == fr.FR_EV_REFUSED]
    whole = {(e.bubble, e.run, e.segment, e.tile0, e.tile1) for e in chunks}
    heads = {(e.bubble, e.run, e.segment, e.tile1) for e in chunks}
    n_whole = n_tail = 0
    for r in refused:
        if (r.bubble, r.run, r.segment, r.tile0, r.tile1) in whole:
            n_whole += 1
        else:
            assert (r.bubble, r.run, r.segment, r.tile0) in heads, "a refused tail follows the tiles its step did"
            n_tail += 1
    assert len(refused) == pr.steps_refused and len(chunks) == pr.steps + n_whole
    whole_refused_work = sum(r.work_units for r in refused if (r.bubble, r.run, r.segment, r.tile0, r.tile1) in whole)
    assert pr.work_units_done == sum(e.work_units for e in chunks) - whole_refused_work
    return n_whole, n_tail


def _oracle_check(got, g, K):
    oracle = pagerank(g.row_ptr, g.col, g.out_degree, 0.85, K)
    assert np.abs(got.astype(np.float64) - oracle).max() <= 1e-5
    big = oracle > 1.0 / g.n_vertices
    assert (np.abs(got[big] - oracle[big]) / oracle[big]).max() <= 1e-4


def test_device_gate_refuses_steps_that_would_start_too_late_and_takes_them_back():
    # The model claims 25 % of the real step times, so the host keeps enqueueing steps that cannot end inside the
    # bubble.  With the device gate each step asks the GPU clock when its kernel starts: the late ones do nothing,
    # are logged, and the task is rewound to the first of them.  The ranks keep the standalone run's bits and are the
    # fp64 oracle's values.
    g = graphs.rmat_csr(21, 1 << 25, seed=9)
    V, E, K = g.n_vertices, g.n_edges, 20
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ref = torch.zeros(V, dtype=torch.float32, device="cuda")
    probe = fr.PageRankTask(V, E, rp, col, od, ref, iterations=K)
    probe.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    ph = probe.fr_pagerank_run_standalone(0, torch.cuda.current_stream(), want_phase_ns=True)
    info = probe.fr_pagerank_info()
    gw, sw = (sum(probe.fr_pagerank_tile_weights(k)) for k in (fr.FR_PR_SEG_GATHER, fr.FR_PR_SEG_SCATTER))
    probe.fr_pagerank_destroy()
    _oracle_check(ref.cpu().numpy(), g, K)
    low = 0.25
    model = _scaled_model(low, ph, K, gw, sw, info)
    stream = torch.cuda.Stream()
    f_ns, b_ns = 1_000_000, 2_000_000
    load = fr.Load(fr.FR_LOAD_BUSYWAIT, fp_ns=f_ns, bp_ns=b_ns)
    late = {}
    for gate in (0, 1):
        ranks = torch.zeros(V, dtype=torch.float32, device="cuda")
        ctx = fr.Context(device_id=0, guard_ns=60_000, launch_cost_ns=5_000, time_steps=4, device_gate=gate)
        task = fr.PageRankTask(V, E, rp, col, od, ranks, iterations=K, max_runs=0, **model)
        tid = ctx.fr_task_register(task.ops, task.user, task.profile)
        assert _init_bubble(ctx, tid) == fr.FR_OK
        stage = fr.Stage(fr.FR_SCHED_1F1B, 4, 8, 2, f_ns, b_ns, load, stream)
        late[gate] = sum(stage.fr_stage_run_epoch(ctx).overruns for _ in range(4))
        import time
        time.sleep(0.05)                                  # the last bubble's verdicts are read once its work has drained
        pr = ctx.fr_query_progress(tid)
        log = ctx.fr_event_log()
        ctx.fr_task_stop(tid)
        got = ranks.cpu().numpy()
        task.fr_pagerank_destroy(); stage.fr_stage_destroy(); ctx.fr_destroy()
        print("gate", gate, "overruns", late[gate], "steps", pr.steps, "refused", pr.steps_refused, "runs", pr.runs_completed, flush=True)
        assert pr.runs_completed >= 1
        assert np.array_equal(got.view(np.uint32), ref.cpu().numpy().view(np.uint32))
        _gate_accounts(log, pr)
        # the work that counts covers the completed runs (and the run in progress, which may have all its gather
        # sweeps behind it and only the finishing pass to go), refused steps excluded
        assert K * E * pr.runs_completed <= pr.work_units_done <= K * E * (pr.runs_completed + 1)
        if gate:
            assert pr.steps_refused > 0
        else:
            assert pr.steps_refused == 0
    load.fr_load_destroy()
    assert late[0] > 0 and late[1] <= late[0], late


def test_device_gate_stops_a_step_between_tiles_and_the_rest_is_taken_up_in_the_next_bubble():
    # On a stream of 8 CUs the sweeps of this graph are hundreds of tiles that the 16 workgroups of a launch hand out
    # among themselves.  The model claims 40 % of the real step times, so steps are still running when their bubble's
    # time is up.  With the device gate the workgroups look at the GPU clock before they take another tile: the step
    # stops after a whole number of its tiles, its record is shortened to those, the rest is logged as refused and
    # done in the next bubble - no step runs past its bubble any more, and the ranks are the standalone run's bits
    # and the fp64 oracle's values.
    K = 4
    g = graphs.fixed_outdeg_csr(1 << 20, 16, seed=34)
    V, E = g.n_vertices, g.n_edges
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ref = torch.zeros(V, dtype=torch.float32, device="cuda")
    side = fr.Context(device_id=0, cu_count=8)
    probe = fr.PageRankTask(V, E, rp, col, od, ref, iterations=K)
    probe.fr_pagerank_run_standalone(0, side.fr_side_stream())
    ph = probe.fr_pagerank_run_standalone(0, side.fr_side_stream(), want_phase_ns=True)
    one = probe.fr_pagerank_run_standalone(0, side.fr_side_stream(), 1, want_phase_ns=True)      # a tile per launch
    info = probe.fr_pagerank_info()
    gw, sw = (sum(probe.fr_pagerank_tile_weights(k)) for k in (fr.FR_PR_SEG_GATHER, fr.FR_PR_SEG_SCATTER))
    probe.fr_pagerank_destroy(); side.fr_destroy()
    _oracle_check(ref.cpu().numpy(), g, K)
    tile_ns = max(one[1] / (K * info.scatter_tiles), one[2] / (K * info.gather_tiles))       # a tile run alone, real time
    low = 0.4
    model = _scaled_model(low, ph, K, gw, sw, info)
    stream = torch.cuda.Stream()
    f_ns, b_ns = 2_000_000, 4_000_000
    load = fr.Load(fr.FR_LOAD_BUSYWAIT, fp_ns=f_ns, bp_ns=b_ns)
    late, tails = {}, {}
    for gate in (0, 1):
        ranks = torch.zeros(V, dtype=torch.float32, device="cuda")
        # the guard covers what the clock checks cannot know: they use the model's tile time, 40 % of the real one, and
        # the tiles of a round run side by side, two workgroups to a compute unit, slower than one alone
        ctx = fr.Context(device_id=0, cu_count=8, guard_ns=int(3 * tile_ns) + 50_000, launch_cost_ns=5_000, time_steps=4, device_gate=gate)
        task = fr.PageRankTask(V, E, rp, col, od, ranks, iterations=K, max_runs=0, **model)
        tid = ctx.fr_task_register(task.ops, task.user, task.profile)
        assert _init_bubble(ctx, tid) == fr.FR_OK
        stage = fr.Stage(fr.FR_SCHED_1F1B, 4, 8, 2, f_ns, b_ns, load, stream)
        late[gate] = 0
        for ep in range(8):
            print("gate", gate, "epoch", ep, flush=True)
            late[gate] += stage.fr_stage_run_epoch(ctx).overruns
        import time
        time.sleep(0.05)
        pr = ctx.fr_query_progress(tid)
        log = ctx.fr_event_log()
        ctx.fr_task_stop(tid)
        got = ranks.cpu().numpy()
        task.fr_pagerank_destroy(); stage.fr_stage_destroy(); ctx.fr_destroy()
        n_whole, tails[gate] = _gate_accounts(log, pr)
        print("gate", gate, "overruns", late[gate], "steps", pr.steps, "refused whole", n_whole, "cut short", tails[gate], "runs", pr.runs_completed, flush=True)
        assert pr.runs_completed >= 1
        assert np.array_equal(got.view(np.uint32), ref.cpu().numpy().view(np.uint32))
        assert K * E * pr.runs_completed <= pr.work_units_done <= K * E * (pr.runs_completed + 1)
    load.fr_load_destroy()
    assert late[0] > 0 and tails[0] == 0
    assert tails[1] > 0 and late[1] == 0, (late, tails)


def test_bubbles_that_end_before_their_declared_end_pause_the_task_and_nothing_is_lost():
    # The paper's online setting: the training system reports a bubble with its expected duration, and the bubble
    # may be over earlier (the next operation's inputs arrived).  Here every bubble is closed after 55 % of its
    # declared length.  The worker stops planning at once; what it had enqueued finishes or is counted as an
    # overrun of the early end, never of the declared one; the task resumes in the next bubble, and a run completed
    # over many such bubbles has the standalone run's bits and the fp64 oracle's values.
    import time
    g = graphs.rmat_csr(18, 1 << 22, seed=15)
    V, E, K = g.n_vertices, g.n_edges, 12
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ref = torch.zeros(V, dtype=torch.float32, device="cuda")
    probe = fr.PageRankTask(V, E, rp, col, od, ref, iterations=K)
    probe.fr_pagerank_run_standalone(0, torch.cuda.current_stream())
    ph = probe.fr_pagerank_run_standalone(0, torch.cuda.current_stream(), want_phase_ns=True)
    info = probe.fr_pagerank_info()
    gw, sw = (sum(probe.fr_pagerank_tile_weights(k)) for k in (fr.FR_PR_SEG_GATHER, fr.FR_PR_SEG_SCATTER))
    probe.fr_pagerank_destroy()
    model = _scaled_model(1.5, ph, K, gw, sw, info)
    ranks = torch.zeros(V, dtype=torch.float32, device="cuda")
    ctx = fr.Context(device_id=0, guard_ns=50_000, launch_cost_ns=5_000, max_chunk_ns=200_000, max_inflight=2, time_steps=1)
    task = fr.PageRankTask(V, E, rp, col, od, ranks, iterations=K, max_runs=1, **model)
    tid = ctx.fr_task_register(task.ops, task.user, task.profile)
    assert _init_bubble(ctx, tid) == fr.FR_OK
    declared, early_ends, late_at_early_end = 2_000_000, 0, 0
    for i in range(400):
        t0 = fr.fr_now_ns()
        ctx.fr_bubble_begin(t0, declared)
        while fr.fr_now_ns() - t0 < 0.55 * declared:
            pass
        rc = ctx.fr_bubble_end()                          # 0.9 ms before the declared end
        assert rc in (fr.FR_OK, fr.FR_ERR_OVERRUN)
        early_ends += 1
        late_at_early_end += rc == fr.FR_ERR_OVERRUN
        while fr.fr_now_ns() - t0 < declared:             # the stage's next operation
            pass
        if ctx.fr_query_progress(tid).runs_completed >= 1:
            break
    time.sleep(0.02)
    pr = ctx.fr_query_progress(tid)
    log = ctx.fr_event_log()
    ctx.fr_task_stop(tid)
    got = ranks.cpu().numpy()
    task.fr_pagerank_destroy(); ctx.fr_destroy()
    print("bubbles", early_ends, "steps", pr.steps, "still running at the early end", late_at_early_end, flush=True)
    assert pr.runs_completed == 1 and pr.bubbles_seen == early_ends + 1
    # a step is at most 0.2 ms of modelled (1.5 x real) time and at most two are in flight: whatever was enqueued when
    # the bubble was closed early is done well before the declared end, 0.9 ms later
    chunks = [e for e in log if e.kind == fr.FR_EV_CHUNK]
    ends = {}
    for e in chunks:
        ends[e.bubble] = max(ends.get(e.bubble, 0), e.t_host_ns + e.measured_ns)
    assert pr.overruns == late_at_early_end
    assert sum(e.work_units for e in chunks) == K * E == pr.work_units_done
    assert np.array_equal(got.view(np.uint32), ref.cpu().numpy().view(np.uint32))
    _oracle_check(got, g, K)


def test_steps_are_timed_in_groups_of_time_steps():
    # time_steps = 3: inside a bubble every third step, and the bubble's last one, carries the GPU time of its group
    import time
    cfg = configs.by_name("cfg1")
    g = cfg.build_graph()
    rp, col, od = _dev(g.row_ptr, torch.int32), _dev(g.col, torch.int32), _dev(g.out_degree, torch.int32)
    ranks = torch.zeros(g.n_vertices, dtype=torch.float32, device="cuda")
    ctx = fr.Context(device_id=0, guard_ns=300_000, launch_cost_ns=25_000, max_chunk_ns=500_000, time_steps=3)
    task = fr.PageRankTask(g.n_vertices, g.n_edges, rp, col, od, ranks, iterations=cfg.iterations, max_runs=2,
                           fs_per_edge=260_000, fs_per_message=400_000, fs_per_vertex=300_000, finish_tile_ns=15000)
    tid = ctx.fr_task_register(task.ops, task.user, task.profile)
    assert _init_bubble(ctx, tid) == fr.FR_OK
    stream = torch.cuda.Stream()
    load = fr.Load(fr.FR_LOAD_BUSYWAIT, fp_ns=cfg.busy_fp_ns, bp_ns=cfg.busy_bp_ns)
    stage = fr.Stage(fr.FR_SCHED_1F1B, cfg.p, cfg.m, cfg.stage, cfg.busy_fp_ns, cfg.busy_bp_ns, load, stream)
    for _ in range(2):
        stage.fr_stage_run_epoch(ctx)
    time.sleep(0.05)
    pr = ctx.fr_query_progress(tid)
    log = ctx.fr_event_log()
    ctx.fr_task_stop(tid)
    task.fr_pagerank_destroy(); stage.fr_stage_destroy(); load.fr_load_destroy(); ctx.fr_destroy()
    by_bubble = {}
    for e in log:
        if e.kind == fr.FR_EV_CHUNK:
            by_bubble.setdefault(e.bubble, []).append(e)
    assert pr.runs_completed == 2 and len(by_bubble) >= 2
    for chunks in by_bubble.values():
        for i, e in enumerate(chunks):
            closes_group = (i + 1) % 3 == 0 or i + 1 == len(chunks)
            assert (e.measured_ns > 0) == closes_group, (i, len(chunks), e.measured_ns)
    total = sum(e.measured_ns for c in by_bubble.values() for e in c)
    assert total == pr.ns_measured and total > 0
