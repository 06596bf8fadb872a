"""Pins for the harvest planner: invariants, boundary cases and a hand-worked example."""
import random

import pytest

from oracle.planner import plan, Record


def test_first_bubble_is_spent_on_init_then_start():
    # Algorithm 2: a CREATED task is initialised by the bubble that finds it; it runs from the next one
    recs = plan([100, 100], [[10, 10]], guard=0, launch_cost=1, max_chunk=1000, max_runs=1)
    assert recs[0] == Record("INIT", 0)
    assert recs[1] == Record("CHUNK", 1, 0, 0, 0, 2, 21)
    assert len(recs) == 2


def test_hand_worked_example():
    # two segments per run: [30, 30, 30] and [50]; guard 10, launch 5, max_chunk 70; bubbles 100, 60, 200
    # bubble 0: budget 90 -> min(90, 70) = 70: 5 + 30 + 30 = 65 fits, + 30 = 95 no -> tiles 0..2, rem 25;
    #           25: 5 + 30 > 25 -> idle 25
    # bubble 1: rem 50: 5 + 30 = 35 -> tile 2..3, rem 15; segment 1: 5 + 50 > 15 -> idle 15
    # bubble 2: rem 190: min(190, 70): 5 + 50 = 55 -> seg 1 done, run 1 starts; rem 135: 65 -> tiles 0..2, rem 70;
    #           35 -> tile 2..3, rem 35; seg 1: 55 > 35 -> idle 35
    recs = plan([100, 60, 200], [[30, 30, 30], [50]], guard=10, launch_cost=5, max_chunk=70, start_created=False)
    assert recs == [
        Record("CHUNK", 0, 0, 0, 0, 2, 65), Record("IDLE", 0, 0, 0, 2, 2, 25),
        Record("CHUNK", 1, 0, 0, 2, 3, 35), Record("IDLE", 1, 0, 1, 0, 0, 15),
        Record("CHUNK", 2, 0, 1, 0, 1, 55), Record("CHUNK", 2, 1, 0, 0, 2, 65),
        Record("CHUNK", 2, 1, 0, 2, 3, 35), Record("IDLE", 2, 1, 1, 0, 0, 35),
    ]


def test_exact_fit_is_allowed_and_one_more_ns_is_not():
    # "only if the remaining time is enough": cost == remaining runs, cost == remaining + 1 idles
    assert plan([100], [[95]], guard=0, launch_cost=5, max_chunk=10**9, max_runs=1, start_created=False)[0].kind == "CHUNK"
    assert plan([99], [[95]], guard=0, launch_cost=5, max_chunk=10**9, max_runs=1, start_created=False)[0].kind == "IDLE"
    # one tile per bubble when the tile fills the bubble exactly
    recs = plan([50, 50, 50], [[40], [40], [40]], guard=5, launch_cost=5, max_chunk=10**9, max_runs=1, start_created=False)
    assert [r.kind for r in recs] == ["CHUNK", "IDLE", "CHUNK", "IDLE", "CHUNK"]
    assert [r.bubble for r in recs if r.kind == "CHUNK"] == [0, 1, 2]


@pytest.mark.parametrize("seed", range(20))
def test_invariants_on_random_inputs(seed):
    rng = random.Random(seed)
    segments = [[rng.randint(1, 50) for _ in range(rng.randint(1, 12))] for _ in range(rng.randint(1, 6))]
    bl = [rng.randint(0, 400) for _ in range(rng.randint(1, 40))]
    guard, launch, max_chunk = rng.randint(0, 20), rng.randint(0, 10), rng.randint(60, 300)
    max_runs = rng.choice([None, 1, 2])
    recs = plan(bl, segments, guard, launch, max_chunk, max_runs)
    assert recs[0] == Record("INIT", 0)
    # chunks walk (run, segment, tile) in order without gaps or repeats, never crossing a segment
    cur = (0, 0, 0)
    used = {}
    for r in recs[1:]:
        assert r.bubble >= 1
        if r.kind == "CHUNK":
            assert (r.run, r.segment, r.tile0) == cur
            assert r.tile0 < r.tile1 <= len(segments[r.segment])
            assert r.modelled_ns == launch + sum(segments[r.segment][r.tile0:r.tile1])
            assert r.modelled_ns <= max_chunk
            used[r.bubble] = used.get(r.bubble, 0) + r.modelled_ns
            assert used[r.bubble] <= bl[r.bubble] - guard      # never past the bubble's end minus the guard
            if r.tile1 == len(segments[r.segment]):
                cur = (r.run + (r.segment + 1 == len(segments)), (r.segment + 1) % len(segments), 0)
            else:
                cur = (r.run, r.segment, r.tile1)
        elif r.kind == "IDLE":
            # idle only when even the next tile alone does not fit
            left = bl[r.bubble] - guard - used.get(r.bubble, 0)
            assert launch + segments[r.segment][r.tile0] > min(left, max_chunk)
    if max_runs is not None:
        assert cur[0] <= max_runs
    # greedy maximality: a chunk stops only at the segment end, at max_chunk/remaining, never earlier
    used = {}
    for r in recs[1:]:
        if r.kind != "CHUNK":
            continue
        left = bl[r.bubble] - guard - used.get(r.bubble, 0)
        if r.tile1 < len(segments[r.segment]):
            assert r.modelled_ns + segments[r.segment][r.tile1] > min(left, max_chunk)
        used[r.bubble] = used.get(r.bubble, 0) + r.modelled_ns


def test_completed_run_covers_every_tile_exactly_once():
    segments = [[7] * 9, [3], [11] * 30, [2] * 4]
    recs = plan([10**6] * 3, segments, guard=0, launch_cost=1, max_chunk=50, max_runs=2)
    seen = {}
    for r in recs:
        if r.kind == "CHUNK":
            for t in range(r.tile0, r.tile1):
                seen[(r.run, r.segment, t)] = seen.get((r.run, r.segment, t), 0) + 1
    want = {(run, g, t) for run in range(2) for g, seg in enumerate(segments) for t in range(len(seg))}
    assert set(seen) == want and set(seen.values()) == {1}


def test_rejects_zero_cost_chunks():
    with pytest.raises(ValueError):
        plan([10], [[0, 0]], guard=0, launch_cost=0, max_chunk=10)


def test_floor_hand_worked_example():
    # one segment [10, 10, 10, 10, 10, 10] with floor 25, second segment [40] with floor 0; launch 5, guard 0
    # bubble 0 (58): step(n) = 5 + max(10 n, 25): n = 5 -> 55 fits, n = 6 -> 65 no -> tiles 0..5 cost 55, rem 3 -> idle
    # bubble 1 (29): step(1) = 5 + max(10, 25) = 30 > 29 -> idle 29: one tile alone is charged the floor
    # bubble 2 (30): step(1) = 30 fits exactly -> tile 5..6 cost 30, rem 0; next segment 45 > 0 -> idle 0
    # bubble 3 (100): segment 1: 45, rem 55; run 1 segment 0: n = 5 -> 55 fits -> rem 0 -> idle 0
    recs = plan([58, 29, 30, 100], [[10] * 6, [40]], guard=0, launch_cost=5, max_chunk=10**9, start_created=False,
                floors=[25, 0])
    assert recs == [
        Record("CHUNK", 0, 0, 0, 0, 5, 55), Record("IDLE", 0, 0, 0, 5, 5, 3),
        Record("IDLE", 1, 0, 0, 5, 5, 29),
        Record("CHUNK", 2, 0, 0, 5, 6, 30), Record("IDLE", 2, 0, 1, 0, 0, 0),
        Record("CHUNK", 3, 0, 1, 0, 1, 45), Record("CHUNK", 3, 1, 0, 0, 5, 55), Record("IDLE", 3, 1, 0, 5, 5, 0),
    ]


def test_zero_floors_change_nothing_and_bad_floors_are_rejected():
    segs, bl = [[30, 30, 30], [50]], [100, 60, 200]
    assert plan(bl, segs, 10, 5, 70, start_created=False) == plan(bl, segs, 10, 5, 70, start_created=False, floors=[0, 0])
    with pytest.raises(ValueError):
        plan(bl, segs, 10, 5, 70, floors=[0])
    with pytest.raises(ValueError):
        plan(bl, segs, 10, 5, 70, floors=[0, -1])


@pytest.mark.parametrize("seed", range(20))
def test_floor_invariants_on_random_inputs(seed):
    # every chunk is charged launch + max(sum, floor), fits its budget, and is maximal: one more tile would not fit
    rng = random.Random(1000 + seed)
    segments = [[rng.randint(1, 50) for _ in range(rng.randint(1, 12))] for _ in range(rng.randint(1, 6))]
    floors = [rng.choice([0, rng.randint(1, 120)]) for _ in segments]
    bl = [rng.randint(0, 400) for _ in range(rng.randint(1, 40))]
    guard, launch, max_chunk = rng.randint(0, 20), rng.randint(0, 10), rng.randint(60, 300)
    recs = plan(bl, segments, guard, launch, max_chunk, None, start_created=False, floors=floors)
    left = {}
    for r in recs:
        rem = left.get(r.bubble, bl[r.bubble] - guard)
        costs = segments[r.segment]
        step = lambda a, b: launch + max(sum(costs[a:b]), floors[r.segment])
        if r.kind == "CHUNK":
            assert r.modelled_ns == step(r.tile0, r.tile1) <= min(rem, max_chunk)
            if r.tile1 < len(costs):
                assert step(r.tile0, r.tile1 + 1) > min(rem, max_chunk)
            left[r.bubble] = rem - r.modelled_ns
        else:
            assert r.kind == "IDLE" and step(r.tile0, r.tile0 + 1) > min(rem, max_chunk)
            assert r.modelled_ns == max(rem, 0)


def test_whole_rounds_rule_hand_worked():
    # one segment of ten tiles of cost 10, three tiles side by side (slots 3), launch 0, no floor.
    # bubble 0: 75 left: seven tiles fit (70), more than a round and short of the segment's end -> six (two whole
    #           rounds, 60); 15 left: one tile (a step of up to `slots` tiles is not cut), 5 left: idle
    # bubble 1: 100 left: the last three tiles reach the segment's end (30); next run: seven fit (70) -> six (60);
    #           10 left: one tile; idle with nothing left
    # without the rule the first step would be the seven tiles
    segs = [[10] * 10]
    recs = plan([75, 100], segs, guard=0, launch_cost=0, max_chunk=10**9, start_created=False, slots=[3])
    assert recs == [
        Record("CHUNK", 0, 0, 0, 0, 6, 60), Record("CHUNK", 0, 0, 0, 6, 7, 10), Record("IDLE", 0, 0, 0, 7, 7, 5),
        Record("CHUNK", 1, 0, 0, 7, 10, 30), Record("CHUNK", 1, 1, 0, 0, 6, 60), Record("CHUNK", 1, 1, 0, 6, 7, 10),
        Record("IDLE", 1, 1, 0, 7, 7, 0),
    ]
    free = plan([75], segs, guard=0, launch_cost=0, max_chunk=10**9, start_created=False)
    assert free[0] == Record("CHUNK", 0, 0, 0, 0, 7, 70)
    # a chunk that reaches the end of its segment is never cut, whatever its length
    recs = plan([1000], segs, guard=0, launch_cost=0, max_chunk=10**9, start_created=False, slots=[3], max_runs=1)
    assert recs == [Record("CHUNK", 0, 0, 0, 0, 10, 100)]


@pytest.mark.parametrize("seed", range(10))
def test_whole_rounds_rule_invariants(seed):
    rng = random.Random(100 + seed)
    segments = [[rng.randint(1, 20) for _ in range(rng.randint(1, 40))] for _ in range(rng.randint(1, 4))]
    slots = [rng.choice([0, 2, 5]) for _ in segments]
    bl = [rng.randint(0, 300) for _ in range(30)]
    recs = plan(bl, segments, guard=3, launch_cost=2, max_chunk=10**9, slots=slots)
    for r in recs:
        if r.kind != "CHUNK":
            continue
        n, s = r.tile1 - r.tile0, slots[r.segment]
        assert r.modelled_ns == 2 + sum(segments[r.segment][r.tile0:r.tile1])
        if s and n > s and r.tile1 < len(segments[r.segment]):
            assert n % s == 0


def test_steps_of_up_to_a_round_hand_worked():
    # One segment of eight tiles of cost 10, four side by side (slots 4), floor 20, launch 0.  A step of n <= 4 tiles is
    # modelled as max(20, 10 n + 20 (4 - n) // 4): 1 -> 25, 2 -> 30, 3 -> 35, 4 -> 40 (a tile alone: its cost and three
    # quarters of the floor; a full round: the sum).
    # bubble 0, 35 left: three tiles fit by the sum (30), and 35 <= 35: three tiles, 35; nothing left: idle
    # bubble 1, 34 left: three fit by the sum but cost 35: two tiles, 30; 4 left: idle
    # bubble 2, 19 left: less than the floor: idle
    # bubble 3, 200 left: tiles 5 .. 7, three tiles: 35; the next run's eight tiles fit and reach the segment's end
    #           (more than a round: the sum, 80); 85 left: eight tiles again, 80; 5 left: idle
    segs = [[10] * 8]
    recs = plan([35, 34, 19, 200], segs, guard=0, launch_cost=0, max_chunk=10**9, start_created=False, floors=[20], slots=[4])
    assert recs == [
        Record("CHUNK", 0, 0, 0, 0, 3, 35), Record("IDLE", 0, 0, 0, 3, 3, 0),
        Record("CHUNK", 1, 0, 0, 3, 5, 30), Record("IDLE", 1, 0, 0, 5, 5, 4),
        Record("IDLE", 2, 0, 0, 5, 5, 19),
        Record("CHUNK", 3, 0, 0, 5, 8, 35), Record("CHUNK", 3, 1, 0, 0, 8, 80), Record("CHUNK", 3, 2, 0, 0, 8, 80),
        Record("IDLE", 3, 3, 0, 0, 0, 5),
    ]
    # no floor: the rule adds nothing; no slots: the old rule, max(sum, floor)
    assert plan([35], segs, guard=0, launch_cost=0, max_chunk=10**9, start_created=False, slots=[4])[0] == Record("CHUNK", 0, 0, 0, 0, 3, 30)
    assert plan([35], segs, guard=0, launch_cost=0, max_chunk=10**9, start_created=False, floors=[20])[0] == Record("CHUNK", 0, 0, 0, 0, 3, 30)
    # a segment of fewer tiles than slots is full with all of them: three tiles of cost 10, slots 8, floor 20:
    # 1 -> 10 + 20 * 2 // 3 = 23, 2 -> 20 + 20 * 1 // 3 = 26, 3 -> 30
    short = [[10] * 3]
    assert plan([25], short, guard=0, launch_cost=0, max_chunk=10**9, start_created=False, floors=[20], slots=[8])[0] == Record("CHUNK", 0, 0, 0, 0, 1, 23)
    assert plan([29], short, guard=0, launch_cost=0, max_chunk=10**9, start_created=False, floors=[20], slots=[8])[0] == Record("CHUNK", 0, 0, 0, 0, 2, 26)
    assert plan([30], short, guard=0, launch_cost=0, max_chunk=10**9, start_created=False, floors=[20], slots=[8])[0] == Record("CHUNK", 0, 0, 0, 0, 3, 30)
    # launch cost counts: 33 left, launch 5: three tiles would be 5 + 35, two are 5 + 30 = 35 > 33, one is 5 + 25 = 30
    assert plan([33], segs, guard=0, launch_cost=5, max_chunk=10**9, start_created=False, floors=[20], slots=[4])[0] == Record("CHUNK", 0, 0, 0, 0, 1, 30)


@pytest.mark.parametrize("seed", range(10))
def test_steps_of_up_to_a_round_invariants(seed):
    rng = random.Random(300 + seed)
    segments = [[rng.randint(1, 20) for _ in range(rng.randint(1, 40))] for _ in range(rng.randint(1, 4))]
    slots = [rng.choice([0, 3, 6]) for _ in segments]
    floors = [rng.choice([0, 7, 25]) for _ in segments]
    bl = [rng.randint(0, 300) for _ in range(40)]
    recs = plan(bl, segments, guard=3, launch_cost=2, max_chunk=10**9, floors=floors, slots=slots)
    remaining = {}
    for r in recs:
        if r.kind == "INIT":
            continue
        rem = remaining.get(r.bubble, bl[r.bubble] - 3)
        if r.kind == "CHUNK":
            n, s, fl = r.tile1 - r.tile0, slots[r.segment], floors[r.segment]
            total = sum(segments[r.segment][r.tile0:r.tile1])
            full = min(s, len(segments[r.segment]))
            want = max(fl, total + fl * (full - n) // full) if s and n <= s else max(total, fl)
            assert r.modelled_ns == 2 + want <= rem
            remaining[r.bubble] = rem - r.modelled_ns
