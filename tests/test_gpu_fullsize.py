"""GPU parity at the configurations' full sizes, in the launch configuration bench.py times: the side task is
harvested inside the bubbles of the GEMM-loaded stage (CU mask and memory cap of the configuration applied), then
compared with the fp64 oracle element by element and, bit for bit, with a standalone run of the same kernels.
Every configuration runs the iteration count it states (the oracle takes about 1, 5, 9 and 45 s for them)."""
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2409_06941_amd as fr          # noqa: E402
from oracle.pagerank import pagerank       # noqa: E402
from workloads import configs              # noqa: E402

# per configuration: iterations, declared FP / BP durations (a little above what the GEMM bursts take), and a cost
# model about twice what the kernels need, so that no step overruns its bubble
CASES = {
    "cfg2": dict(K=50, f_ns=4_500_000, b_ns=9_000_000, epochs=3,
                 model=dict(fs_per_edge=2000, fs_per_message=3000, fs_per_vertex=2000, finish_tile_ns=200,
                            min_step_ns=(30_000, 100_000, 100_000, 30_000))),
    "cfg3": dict(K=50, f_ns=4_500_000, b_ns=9_000_000, epochs=4,
                 model=dict(fs_per_edge=2500, fs_per_message=3500, fs_per_vertex=4000, finish_tile_ns=200,
                            min_step_ns=(30_000, 150_000, 100_000, 30_000))),
    "cfg4": dict(K=100, f_ns=4_500_000, b_ns=9_000_000, epochs=6,
                 model=dict(fs_per_edge=6000, fs_per_message=8000, fs_per_vertex=12000, finish_tile_ns=500,
                            min_step_ns=(30_000, 300_000, 200_000, 50_000))),
    "cfg5": dict(K=100, f_ns=36_000_000, b_ns=72_000_000, epochs=2,
                 model=dict(fs_per_edge=2500, fs_per_message=5000, fs_per_vertex=4000, finish_tile_ns=200,
                            min_step_ns=(30_000, 300_000, 100_000, 30_000))),
}


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4", "cfg5"])
def test_full_size_harvested_run_matches_oracle_and_standalone_bits(name):
    cfg = configs.by_name(name)
    case = CASES[name]
    print("building %s graph" % name, flush=True)
    g = cfg.build_graph()
    V, E, K = g.n_vertices, g.n_edges, case["K"]
    mem_cap = cfg.mem_cap_bytes if cfg.mem_cap_bytes else (64 << 30)
    cu_count = cfg.cu_count if cfg.cu_count < 256 else 0
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    rp, col, od = dev(g.row_ptr), dev(g.col), dev(g.out_degree)
    ref = torch.zeros(V, dtype=torch.float32, device="cuda")
    ranks = torch.zeros(V, dtype=torch.float32, device="cuda")

    # (on a stream with the configuration's CU mask: the layout is cut for the compute units of the stream it is built
    # on, and a range cut into several pieces adds its partial sums in fp32, so bits are only the same per CU count)
    print("standalone run, 37 tiles per launch", flush=True)
    probe = fr.Context(device_id=0, cu_count=cu_count)
    t = fr.PageRankTask(V, E, rp, col, od, ref, damping=cfg.damping, iterations=K, mem_limit_bytes=mem_cap)
    t.fr_pagerank_run_standalone(0, probe.fr_side_stream(), 37)
    info = t.fr_pagerank_info()
    t.fr_pagerank_destroy()
    probe.fr_destroy()
    assert info.bytes_resident <= info.bytes_peak <= mem_cap            # set-up scratch included

    print("harvested run beside the GEMM stage load", flush=True)
    L = cfg.load
    stream = torch.cuda.Stream()
    ws = torch.empty(fr.Load.fr_load_workspace_bytes(fr.FR_LOAD_GPT, L.layers, L.hidden, L.ffn, L.tokens), dtype=torch.uint8, device="cuda")
    load = fr.Load(fr.FR_LOAD_GPT, L.layers, L.hidden, L.ffn, L.tokens, workspace=ws, seed=cfg.seed, stream=stream)
    ctx = fr.Context(device_id=0, cu_count=cu_count, guard_ns=300_000, launch_cost_ns=10_000, time_steps=1,
                     mem_available_bytes=mem_cap + 1)
    task = fr.PageRankTask(V, E, rp, col, od, ranks, damping=cfg.damping, iterations=K, max_runs=1, mem_limit_bytes=mem_cap,
                           **case["model"])
    tid = ctx.fr_task_register(task.ops, task.user, task.profile)
    ctx.fr_bubble_begin(fr.fr_now_ns(), 5_000_000_000)
    t_end = time.time() + 60
    while ctx.fr_query_progress(tid).state == fr.FR_CREATED and time.time() < t_end:
        time.sleep(0.001)
    assert ctx.fr_bubble_end() == fr.FR_OK
    sched = fr.FR_SCHED_1F1B if cfg.schedule == "1f1b" else fr.FR_SCHED_GPIPE
    stage = fr.Stage(sched, cfg.p, cfg.m, cfg.stage, case["f_ns"], case["b_ns"], load, stream)
    for ep in range(case["epochs"]):
        print("epoch", ep, flush=True)
        stage.fr_stage_run_epoch(ctx)
        if ctx.fr_query_progress(tid).runs_completed >= 1:
            break
    pr = ctx.fr_query_progress(tid)
    log = ctx.fr_event_log()
    ctx.fr_task_stop(tid)
    got = ranks.cpu().numpy()
    ref_bits = ref.cpu().numpy()
    task.fr_pagerank_destroy(); stage.fr_stage_destroy(); load.fr_load_destroy(); ctx.fr_destroy()

    assert pr.runs_completed == 1 and pr.overruns == 0
    assert sum(e.work_units for e in log if e.kind == fr.FR_EV_CHUNK) == K * E
    assert np.array_equal(got.view(np.uint32), ref_bits.view(np.uint32))

    print("oracle", flush=True)
    want = pagerank(g.row_ptr, g.col, g.out_degree, cfg.damping, K)
    err = np.abs(got.astype(np.float64) - want)
    assert err.max() <= 1e-5
    big = want > 1.0 / V
    assert (err[big] / want[big]).max() <= 1e-4
    assert abs(float(got.astype(np.float64).sum()) - 1.0) <= 1e-4
