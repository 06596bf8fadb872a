"""CPU oracle: which side-task work lands in which bubble.  Test infrastructure only.

Follows the paper's bubble/side-task management loop for one worker serving one task (Section 4.4,
Algorithm 2) and its program-directed time limit (Section 4.5):

  * when a new bubble arrives and the current task is CREATED, the manager initialises it (-> PAUSED); that
    bubble is spent on initialisation.  When the task is PAUSED, the manager starts it (-> RUNNING) and hands
    it the bubble's end time;
  * while RUNNING, before each step the task checks that the time left in the bubble is enough for the step
    and runs the step only then; otherwise the rest of the bubble stays idle (the "insufficient time" share of
    the paper's bubble-time breakdown, Section 6.5);
  * when the bubble ends the task is paused.

A "step" here is a chunk: a run of consecutive tiles of the task's current segment.  The task's work is a fixed
sequence of segments (for PageRank: the phases of each iteration, in order); a chunk never spans two segments.
Costs are modelled integer nanoseconds known up front, so the whole plan is a pure function of the declared
bubble lengths and the cost table -- no clock is read.

    remaining = L_i - guard
    repeat:
        step(n) = launch_cost + max(sum of the next n tile costs, floor of the segment)
        n = the largest count of consecutive tiles from the cursor, inside the current segment, with
            step(n) <= min(remaining, max_chunk)
        n == 0  ->  idle for the rest of the bubble
        else    ->  run the chunk; remaining -= step(n); advance the cursor

The floor is the profiled duration of the segment's shortest step (Section 4.3 profiles the per-step duration):
tiles of one step run side by side on the GPU, so a step of a few tiles is not shorter than a step of one.

Rounds (optional, per segment): a task may say that at most `slots` tiles of a segment run side by side and that a
step of more tiles runs in rounds, its modelled cost - the sum - being what whole rounds take.  Section 4.5 lets a
step run only if the time left is enough for it, so a step must not take longer than modelled: a chunk of more
than `slots` tiles that does not reach the segment's end is cut down to a whole number of rounds,
n -> (n // slots) * slots (a round and a few tiles would take two rounds' time).  A step of up to one round runs its
tiles side by side on part of the slots: one tile alone takes the floor, a full round the sum of its tile costs, and
in between the time grows with the number of tiles, so such a step is modelled as
    max(floor, sum of its n tile costs + floor * (full - n) // full),   full = min(slots, tiles of the segment)
and n is taken down until that fits.  slots = 0: neither rule.

When the last segment of a run completes the task starts over (run index + 1) unless `max_runs` is reached,
after which it harvests nothing more.
"""
from dataclasses import dataclass
from typing import List, Optional, Sequence


@dataclass(frozen=True)
class Record:
    kind: str          # "INIT", "CHUNK", "IDLE"
    bubble: int
    run: int = 0
    segment: int = 0   # index into the segment list of one run
    tile0: int = 0
    tile1: int = 0
    modelled_ns: int = 0   # CHUNK: launch_cost + max(sum of tile costs, floor); IDLE: modelled time left unused


def plan(bubble_lengths: Sequence[int], segments: Sequence[Sequence[int]], guard: int, launch_cost: int,
         max_chunk: int, max_runs: Optional[int] = None, start_created: bool = True,
         floors: Optional[Sequence[int]] = None, slots: Optional[Sequence[int]] = None) -> List[Record]:
    """Plan over the given bubbles.  segments[g][t] is the modelled cost of tile t of segment g (ints >= 0);
    floors[g] (default 0) is the least modelled cost of any step of segment g; slots[g] (default 0 = no rule) is the
    number of tiles of segment g that run side by side (see "Rounds" above).

    start_created: the task begins in CREATED, so the first bubble is consumed by initialisation.
    """
    if floors is None:
        floors = [0] * len(segments)
    if len(floors) != len(segments) or any(f < 0 for f in floors):
        raise ValueError("one non-negative floor per segment")
    if slots is None:
        slots = [0] * len(segments)
    if len(slots) != len(segments) or any(x < 0 for x in slots):
        raise ValueError("one non-negative slot count per segment")
    if launch_cost < 0 or guard < 0 or max_chunk <= 0:
        raise ValueError("bad planner constants")
    if any(len(seg) == 0 for seg in segments) or len(segments) == 0:
        raise ValueError("every segment needs at least one tile")
    if launch_cost == 0 and any(c <= 0 for seg in segments for c in seg):
        raise ValueError("a chunk must have a positive modelled cost")
    out: List[Record] = []
    created = start_created
    run, seg, tile = 0, 0, 0
    for i, length in enumerate(bubble_lengths):
        if created:
            created = False
            out.append(Record("INIT", i))
            continue
        remaining = length - guard
        while True:
            if max_runs is not None and run >= max_runs:
                break                                   # task finished: nothing left to harvest
            budget = min(remaining, max_chunk)
            costs = segments[seg]
            n, tiles_cost = 0, 0
            while tile + n < len(costs) and launch_cost + max(tiles_cost + costs[tile + n], floors[seg]) <= budget:
                tiles_cost += costs[tile + n]
                n += 1
            if slots[seg] and n > slots[seg] and tile + n < len(costs):
                n = n // slots[seg] * slots[seg]
                tiles_cost = sum(costs[tile:tile + n])
            total = launch_cost + max(tiles_cost, floors[seg])
            if slots[seg] and 0 < n <= slots[seg]:
                full = min(slots[seg], len(costs))          # a segment of fewer tiles than slots is full with all of them

                def part(k):
                    return max(floors[seg], sum(costs[tile:tile + k]) + floors[seg] * (full - k) // full)
                while n > 0 and launch_cost + part(n) > budget:
                    n -= 1
                if n > 0:
                    tiles_cost = sum(costs[tile:tile + n])
                    total = launch_cost + part(n)
            if n == 0:
                out.append(Record("IDLE", i, run, seg, tile, tile, max(remaining, 0)))
                break
            out.append(Record("CHUNK", i, run, seg, tile, tile + n, total))
            remaining -= total
            tile += n
            if tile == len(costs):
                tile = 0
                seg += 1
                if seg == len(segments):
                    seg = 0
                    run += 1
    return out
