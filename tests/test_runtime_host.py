"""Host-side runtime tests on a host-only context (device_id = -1): no GPU call is made.

The fake task below enqueues nothing; it only plans steps from a cost table, like the PageRank task does, so the
runtime's state machine, admission test, memory limit, bubble protocol and step loop can be checked against the
CPU oracle of the harvest plan.
"""
import ctypes as C
import time

import pytest

import paper_2409_06941_amd as fr
from oracle import planner


class FakeTask:
    """A task over `segments` (lists of tile costs) that restarts after the last segment."""

    def __init__(self, segments, max_runs=0, init_alloc=(), init_rc=0, charge=0):
        self.segments = segments
        self.max_runs = max_runs
        self.init_alloc = init_alloc
        self.init_rc = init_rc
        self.charge = charge
        self.run = self.seg = self.tile = 0
        self.calls = []
        self.alloc_results = []
        self.ops = fr.fr_task_ops(fr.binding.CREATE_FN(self._create), fr.binding.INIT_FN(self._init),
                                  fr.binding.PLAN_FN(self._plan), fr.binding.RUN_FN(self._run),
                                  fr.binding.STOP_FN(self._stop))

    def _create(self, user):
        self.calls.append("create")
        return 0

    def _init(self, user, alloc, stream):
        self.calls.append("init")
        if self.charge:
            fr.lib().fr_alloc_charge(alloc, self.charge)
        for n in self.init_alloc:
            self.alloc_results.append(fr.lib().fr_alloc_device(alloc, n))
        return self.init_rc

    def _plan(self, user, budget, launch, out):
        st = out.contents
        st.modelled_ns = 0; st.work_units = 0; st.finished = 0; st.completes_run = 0
        st.run, st.segment, st.tile0, st.tile1 = self.run, self.seg, self.tile, self.tile
        if self.max_runs and self.run >= self.max_runs:
            st.finished = 1
            return 0
        costs = self.segments[self.seg]
        prefix = [0]
        for c in costs:
            prefix.append(prefix[-1] + c)
        n = fr.fr_chunk_fit(prefix, self.tile, budget, launch)
        if n:
            st.tile1 = self.tile + n
            st.modelled_ns = prefix[self.tile + n] - prefix[self.tile]
            st.work_units = n
            st.completes_run = int(self.seg + 1 == len(self.segments) and st.tile1 == len(costs))
        return 0

    def _run(self, user, stream, planned):
        st = planned.contents
        self.calls.append(("run", st.run, st.segment, st.tile0, st.tile1))
        self.tile = st.tile1
        if self.tile == len(self.segments[self.seg]):
            self.tile = 0
            self.seg += 1
            if self.seg == len(self.segments):
                self.seg = 0
                self.run += 1
        return 0

    def _stop(self, user):
        self.calls.append("stop")
        return 0


def _bubble(ctx, length_ns, hold_s=0.004):
    ctx.fr_bubble_begin(fr.fr_now_ns(), length_ns)
    time.sleep(hold_s)
    return ctx.fr_bubble_end()


def _log(ctx):
    names = {fr.FR_EV_INIT: "INIT", fr.FR_EV_CHUNK: "CHUNK", fr.FR_EV_IDLE: "IDLE", fr.FR_EV_MISS: "MISS", fr.FR_EV_OVERRUN: "OVERRUN"}
    return [(names[e.kind], e.bubble, e.run, e.segment, e.tile0, e.tile1, e.modelled_ns) for e in ctx.fr_event_log()]


def _oracle_log(recs):
    out = []
    for r in recs:
        if r.kind == "INIT":
            out.append(("INIT", r.bubble, 0, 0, 0, 0, 0))
        else:
            out.append((r.kind, r.bubble, r.run, r.segment, r.tile0, r.tile1, r.modelled_ns))
    return out


@pytest.fixture
def ctx():
    c = fr.Context(device_id=-1, mem_available_bytes=1000, guard_ns=0, launch_cost_ns=0)
    yield c
    c.fr_destroy()


def test_admission_needs_strictly_more_free_memory_than_the_task_asks(ctx):
    # Algorithm 1: a worker qualifies only if its free memory exceeds the task's requirement
    t = FakeTask([[1]])
    with pytest.raises(fr.FreeRideError) as e:
        ctx.fr_task_register(t.ops, None, fr.fr_task_profile(1000, 1))
    assert e.value.code == fr.FR_ERR_NOMEM and t.calls == []
    tid = ctx.fr_task_register(t.ops, None, fr.fr_task_profile(999, 1))
    assert t.calls == ["create"]
    assert ctx.fr_query_progress(tid).state == fr.FR_CREATED
    # Algorithm 1 looks at the worker's free memory only: a second accepted task waits in the worker's queue
    t2 = FakeTask([[1]])
    tid2 = ctx.fr_task_register(t2.ops, None, fr.fr_task_profile(10, 1))
    assert ctx.fr_query_progress(tid2).state == fr.FR_SUBMITTED and t2.calls == []
    with pytest.raises(fr.FreeRideError) as e:
        ctx.fr_task_register(t2.ops, None, fr.fr_task_profile(1000, 1))
    assert e.value.code == fr.FR_ERR_NOMEM


def test_state_walk_created_paused_running_paused_stopped(ctx):
    t = FakeTask([[1000, 1000]], max_runs=1)
    tid = ctx.fr_task_register(t.ops, None, fr.fr_task_profile(10, 1))
    assert _bubble(ctx, 10_000_000_000) == fr.FR_OK             # first bubble: InitSideTask only
    assert ctx.fr_query_progress(tid).state == fr.FR_PAUSED and t.calls == ["create", "init"]
    ctx.fr_bubble_begin(fr.fr_now_ns(), 10_000_000_000)
    deadline = time.time() + 5
    while ctx.fr_query_progress(tid).steps == 0 and time.time() < deadline:
        time.sleep(0.001)
    pr = ctx.fr_query_progress(tid)
    assert pr.steps == 1 and pr.runs_completed == 1
    ctx.fr_bubble_end()
    assert ctx.fr_query_progress(tid).state == fr.FR_PAUSED      # PauseSideTask at the bubble's end
    assert ctx.fr_task_stop(tid) == fr.FR_OK
    assert ctx.fr_query_progress(tid).state == fr.FR_STOPPED and t.calls[-1] == "stop"
    with pytest.raises(fr.FreeRideError) as e:
        ctx.fr_task_stop(tid)
    assert e.value.code == fr.FR_ERR_STATE
    _bubble(ctx, 10_000_000_000)                                 # a stopped task is never served again
    assert t.calls[-1] == "stop"


def test_stop_is_legal_from_created(ctx):
    t = FakeTask([[1]])
    tid = ctx.fr_task_register(t.ops, None, fr.fr_task_profile(10, 1))
    assert ctx.fr_task_stop(tid) == fr.FR_OK
    assert t.calls == ["create", "stop"]
    # the context can take a new task afterwards
    t2 = FakeTask([[1]])
    ctx.fr_task_register(t2.ops, None, fr.fr_task_profile(10, 1))


def test_bubble_protocol_errors(ctx):
    with pytest.raises(fr.FreeRideError) as e:
        ctx.fr_bubble_end()
    assert e.value.code == fr.FR_ERR_STATE
    ctx.fr_bubble_begin(fr.fr_now_ns(), 1000)
    with pytest.raises(fr.FreeRideError) as e:
        ctx.fr_bubble_begin(fr.fr_now_ns(), 1000)
    assert e.value.code == fr.FR_ERR_STATE
    assert ctx.fr_bubble_end() == fr.FR_OK


def test_memory_limit_stops_only_the_task(ctx):
    # the task may take 600 bytes; 256 + 256 fit (rounded to 256), the third request passes the limit
    t = FakeTask([[1]], init_alloc=(200, 256, 1))
    tid = ctx.fr_task_register(t.ops, None, fr.fr_task_profile(600, 1))
    assert _bubble(ctx, 1_000_000_000) == fr.FR_OK
    pr = ctx.fr_query_progress(tid)
    assert pr.state == fr.FR_STOPPED and pr.last_error == fr.FR_ERR_OOM
    assert t.alloc_results[0] and t.alloc_results[1] and not t.alloc_results[2]
    assert t.calls == ["create", "init", "stop"]
    assert _bubble(ctx, 1_000_000) == fr.FR_OK                   # the stage's bubbles go on undisturbed


def test_charged_caller_buffers_count_against_the_limit(ctx):
    t = FakeTask([[1]], charge=500, init_alloc=(256,))
    tid = ctx.fr_task_register(t.ops, None, fr.fr_task_profile(700, 1))
    _bubble(ctx, 1_000_000_000)
    pr = ctx.fr_query_progress(tid)
    assert pr.state == fr.FR_STOPPED and pr.last_error == fr.FR_ERR_OOM


def test_failed_init_stops_the_task(ctx):
    t = FakeTask([[1]], init_rc=fr.FR_ERR_ARG)
    tid = ctx.fr_task_register(t.ops, None, fr.fr_task_profile(10, 1))
    _bubble(ctx, 1_000_000_000)
    pr = ctx.fr_query_progress(tid)
    assert pr.state == fr.FR_STOPPED and pr.last_error == fr.FR_ERR_ARG


@pytest.mark.parametrize("guard,launch,max_chunk", [(0, 0, 0), (7, 3, 0), (5, 2, 120)])
def test_paused_mid_plan_keeps_the_cursor_and_the_cost_rule(guard, launch, max_chunk):
    # Bubbles are declared far longer than they are held open, so fr_bubble_end pauses the task while the plan
    # still has budget.  Whatever was enqueued must continue exactly where the previous bubble stopped, and every
    # step's modelled cost must be launch_cost + the sum of its tiles.
    ms = 1_000_000
    segments = [[30, 45, 20, 5], [60], [10] * 9, [33, 33]]
    c = fr.Context(device_id=-1, guard_ns=guard * ms, launch_cost_ns=launch * ms, max_chunk_ns=max_chunk * ms)
    t = FakeTask([[x * ms for x in seg] for seg in segments])
    c.fr_task_register(t.ops, None, fr.fr_task_profile(10, 1))
    for L in [100, 100, 64, 300, 12, 250, 0, 90]:
        _bubble(c, L * ms * 1000, hold_s=0.003)
    got = _log(c)
    c.fr_destroy()
    assert got[0] == ("INIT", 0, 0, 0, 0, 0, 0)
    cur = (0, 0, 0)
    n_chunks = 0
    for kind, bubble, run, seg, t0, t1, cost in got[1:]:
        assert bubble >= 1
        if kind != "CHUNK":
            continue
        n_chunks += 1
        assert (run, seg, t0) == cur
        tiles = segments[seg]
        assert cost == (launch + sum(tiles[t0:t1])) * ms
        if max_chunk:
            assert cost <= max_chunk * ms
        if t1 == len(tiles):
            cur = (run + (seg + 1 == len(segments)), (seg + 1) % len(segments), 0)
        else:
            cur = (run, seg, t1)
    assert n_chunks > 10


def test_exact_plan_match_with_tight_bubbles():
    # Declared lengths equal to what the model uses: the whole log must equal the oracle's plan exactly.
    ms = 1_000_000
    segments = [[3 * ms, 4 * ms, 2 * ms], [6 * ms], [1 * ms] * 5]
    lengths = [20 * ms, 9 * ms, 14 * ms, 3 * ms, 30 * ms, 11 * ms]
    guard, launch, max_chunk = 1 * ms, ms // 2, 8 * ms
    c = fr.Context(device_id=-1, guard_ns=guard, launch_cost_ns=launch, max_chunk_ns=max_chunk)
    t = FakeTask(segments, max_runs=2)
    c.fr_task_register(t.ops, None, fr.fr_task_profile(10, 1))
    for L in lengths:
        c.fr_bubble_begin(fr.fr_now_ns(), L)
        time.sleep(L / 1e9 + 0.002)
        c.fr_bubble_end()
    got = _log(c)
    c.fr_destroy()
    want = _oracle_log(planner.plan(lengths, segments, guard, launch, max_chunk, max_runs=2))
    assert got == want


def test_late_notification_is_a_deadline_miss_not_an_overrun():
    # the bubble is reported as having begun long ago: the model says the step fits, the clock says it does not
    ms = 1_000_000
    c = fr.Context(device_id=-1, guard_ns=0, launch_cost_ns=0)
    t = FakeTask([[5 * ms]])
    tid = c.fr_task_register(t.ops, None, fr.fr_task_profile(10, 1))
    _bubble(c, 10 * ms)
    c.fr_bubble_begin(fr.fr_now_ns() - 8 * ms, 10 * ms)          # 2 ms really left, step needs 5
    time.sleep(0.003)
    c.fr_bubble_end()
    pr = c.fr_query_progress(tid)
    log = _log(c)
    c.fr_destroy()
    assert pr.deadline_misses == 1 and pr.steps == 0
    assert log[-1][0] == "MISS"


def test_init_that_outlives_its_bubble_does_not_hold_the_stage():
    # InitSideTask is protected like any step (Section 4.5): when it is still running at the bubble's end the
    # stage is not made to wait; the call reports an overrun and the task starts running in a later bubble.
    ms = 1_000_000

    class SlowInit(FakeTask):
        def _init(self, user, alloc, stream):
            time.sleep(0.08)
            return super()._init(user, alloc, stream)

    c = fr.Context(device_id=-1, guard_ns=0, launch_cost_ns=0)
    t = SlowInit([[1 * ms]], max_runs=1)
    t.ops = fr.fr_task_ops(fr.binding.CREATE_FN(t._create), fr.binding.INIT_FN(t._init), fr.binding.PLAN_FN(t._plan),
                           fr.binding.RUN_FN(t._run), fr.binding.STOP_FN(t._stop))
    tid = c.fr_task_register(t.ops, None, fr.fr_task_profile(10, 1))
    c.fr_bubble_begin(fr.fr_now_ns(), 5 * ms)
    time.sleep(0.005)
    t0 = time.time()
    assert c.fr_bubble_end() == fr.FR_ERR_OVERRUN
    assert time.time() - t0 < 0.02                                  # returned at once
    assert c.fr_query_progress(tid).state == fr.FR_CREATED
    time.sleep(0.12)                                                # init finishes between bubbles
    assert c.fr_query_progress(tid).state == fr.FR_PAUSED
    assert _bubble(c, 50 * ms, hold_s=0.01) == fr.FR_OK
    pr = c.fr_query_progress(tid)
    c.fr_destroy()
    assert pr.overruns == 1 and pr.runs_completed == 1


def test_queued_tasks_take_over_in_order_when_the_current_one_finishes_or_stops():
    # Algorithms 1 and 2: accepted tasks queue up on the worker; the head becomes current (created) when the worker
    # has no live task, is initialised by the next bubble and runs from the one after
    ms = 1_000_000
    c = fr.Context(device_id=-1, guard_ns=0, launch_cost_ns=0)
    a, b, d = FakeTask([[1 * ms, 1 * ms]], max_runs=1), FakeTask([[1 * ms]], max_runs=0), FakeTask([[1 * ms]], max_runs=1)
    ia = c.fr_task_register(a.ops, None, fr.fr_task_profile(10, 1))
    ib = c.fr_task_register(b.ops, None, fr.fr_task_profile(10, 1))
    idd = c.fr_task_register(d.ops, None, fr.fr_task_profile(10, 1))
    assert [c.fr_query_progress(i).state for i in (ia, ib, idd)] == [fr.FR_CREATED, fr.FR_SUBMITTED, fr.FR_SUBMITTED]
    assert _bubble(c, 10 * ms) == fr.FR_OK                      # a: init
    assert _bubble(c, 10 * ms) == fr.FR_OK                      # a: both tiles, then finished -> b becomes current
    pa = c.fr_query_progress(ia)
    assert pa.state == fr.FR_STOPPED and pa.runs_completed == 1 and pa.last_error == fr.FR_OK and a.calls[-1] == "stop"
    assert c.fr_query_progress(ib).state == fr.FR_CREATED and b.calls == ["create"]
    assert _bubble(c, 10 * ms) == fr.FR_OK                      # b: init
    assert _bubble(c, 3 * ms + 1) == fr.FR_OK                   # b: three one-tile runs
    assert c.fr_query_progress(ib).runs_completed == 3 and c.fr_query_progress(idd).state == fr.FR_SUBMITTED
    c.fr_task_stop(ib)                                          # b never finishes by itself; stopping it promotes d
    assert c.fr_query_progress(ib).state == fr.FR_STOPPED and c.fr_query_progress(idd).state == fr.FR_CREATED
    assert _bubble(c, 10 * ms) == fr.FR_OK and _bubble(c, 10 * ms) == fr.FR_OK
    pd = c.fr_query_progress(idd)
    assert pd.runs_completed == 1 and pd.state == fr.FR_PAUSED   # finished with nobody waiting: stays paused
    c.fr_destroy()
    assert d.calls[-1] == "stop"


def test_a_queued_task_can_be_withdrawn():
    c = fr.Context(device_id=-1)
    a, b = FakeTask([[1]]), FakeTask([[1]])
    ia = c.fr_task_register(a.ops, None, fr.fr_task_profile(10, 1))
    ib = c.fr_task_register(b.ops, None, fr.fr_task_profile(10, 1))
    c.fr_task_stop(ib)
    assert c.fr_query_progress(ib).state == fr.FR_STOPPED and b.calls == []          # never created, never stopped
    with pytest.raises(fr.FreeRideError) as e:
        c.fr_task_stop(ib)
    assert e.value.code == fr.FR_ERR_STATE
    c.fr_task_stop(ia)
    assert c.fr_query_progress(ia).state == fr.FR_STOPPED
    c.fr_destroy()


class _SlowRun(FakeTask):
    """A task whose run_step does not return for `sleep_s` (a misbehaving side task, Section 4.5)."""
    sleep_s = 0.08

    def _run(self, user, stream, planned):
        time.sleep(self.sleep_s)
        return super()._run(user, stream, planned)


def _slow(cls, *args, **kw):
    t = cls(*args, **kw)
    t.ops = fr.fr_task_ops(fr.binding.CREATE_FN(t._create), fr.binding.INIT_FN(t._init), fr.binding.PLAN_FN(t._plan),
                           fr.binding.RUN_FN(t._run), fr.binding.STOP_FN(t._stop))
    return t


@pytest.mark.parametrize("grace_ms,killed", [(10, True), (0, False), (500, False)])
def test_framework_enforced_limit_stops_a_task_whose_step_does_not_return(grace_ms, killed):
    # the stage is never held up by the late callback; once the grace period is over the task is stopped (the
    # paper's worker kills the process) and the next task in the queue takes over
    ms = 1_000_000
    c = fr.Context(device_id=-1, guard_ns=0, launch_cost_ns=0, grace_ns=grace_ms * ms)
    bad, good = _slow(_SlowRun, [[1 * ms]]), FakeTask([[1 * ms]], max_runs=1)
    ib = c.fr_task_register(bad.ops, None, fr.fr_task_profile(10, 1))
    ig = c.fr_task_register(good.ops, None, fr.fr_task_profile(10, 1))
    assert _bubble(c, 10 * ms) == fr.FR_OK                      # init
    c.fr_bubble_begin(fr.fr_now_ns(), 5 * ms)
    time.sleep(0.005)
    t0 = time.time()
    assert c.fr_bubble_end() == fr.FR_ERR_OVERRUN               # run_step is still asleep
    assert time.time() - t0 < 0.02
    assert c.fr_query_progress(ib).state == fr.FR_RUNNING
    time.sleep(0.03)                                            # past a 10 ms grace period, callback still asleep
    c.fr_bubble_begin(fr.fr_now_ns(), 1 * ms)                   # the check happens at bubble notifications
    time.sleep(0.001)
    c.fr_bubble_end()
    time.sleep(0.1)                                             # the callback returns; the worker acts on the verdict
    pb = c.fr_query_progress(ib)
    if killed:
        assert pb.state == fr.FR_STOPPED and pb.last_error == fr.FR_ERR_OVERRUN and pb.killed == 1
        assert bad.calls[-1] == "stop"
        # the queue moves on (the worker may already have served the short bubble late and initialised the next task)
        assert c.fr_query_progress(ig).state in (fr.FR_CREATED, fr.FR_PAUSED) and good.calls[0] == "create"
    else:
        assert pb.state == fr.FR_PAUSED and pb.killed == 0 and pb.overruns >= 1
        assert c.fr_query_progress(ig).state == fr.FR_SUBMITTED
    c.fr_destroy()


def test_framework_enforced_limit_covers_initialisation():
    ms = 1_000_000

    class SlowInit(FakeTask):
        def _init(self, user, alloc, stream):
            time.sleep(0.08)
            return super()._init(user, alloc, stream)

    c = fr.Context(device_id=-1, guard_ns=0, launch_cost_ns=0, grace_ns=10 * ms)
    t = _slow(SlowInit, [[1 * ms]])
    tid = c.fr_task_register(t.ops, None, fr.fr_task_profile(10, 1))
    c.fr_bubble_begin(fr.fr_now_ns(), 5 * ms)
    time.sleep(0.005)
    assert c.fr_bubble_end() == fr.FR_ERR_OVERRUN
    time.sleep(0.03)
    c.fr_bubble_begin(fr.fr_now_ns(), 1 * ms)
    time.sleep(0.001)
    c.fr_bubble_end()
    time.sleep(0.1)
    pr = c.fr_query_progress(tid)
    c.fr_destroy()
    assert pr.state == fr.FR_STOPPED and pr.last_error == fr.FR_ERR_OVERRUN and pr.killed == 1


def test_cost_scale_update_rule():
    # rises at once (at most doubling per step), falls by an eighth of the gap per step, stays within [0.25, 16],
    # ignores steps without a model
    nxt = fr.binding.fr_cost_scale_next
    assert nxt(1_000_000, 100, 150) == 1_500_000
    assert nxt(1_000_000, 100, 250) == 2_000_000 and nxt(2_000_000, 100, 250) == 2_500_000
    assert nxt(2_500_000, 100, 100) == 2_500_000 - 1_500_000 // 8 == 2_312_500
    assert nxt(1_000_000, 100, 1) == 1_000_000 - 750_000 // 8
    assert nxt(1_000_000, 0, 5) == 1_000_000
    assert nxt(1_000_000, 1, 10**9) == 2_000_000 and nxt(12_000_000, 1, 10**9) == 16_000_000
    assert nxt(10, 100, 100) == 500_000                     # an out-of-range scale is clamped (to 0.25) first, then doubles
    s, seen = 4_000_000, []
    for _ in range(200):                                    # constant ratio 1.3: monotone decay towards it, never below
        s = nxt(s, 1000, 1300)
        seen.append(s)
    assert all(a >= b for a, b in zip(seen, seen[1:])) and 1_300_000 <= seen[-1] <= 1_300_010
