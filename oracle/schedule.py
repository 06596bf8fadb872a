"""CPU oracle: pipeline schedule simulator that yields one stage's bubble windows.  Test infrastructure only.

Follows the paper's description of pipeline training (Section 2.1): every micro-batch undergoes a forward
pass (FP) and a backward pass (BP) on every stage; a stage hands its output to its neighbour and moves on to its
next operation at once; bubbles are the periods a stage idles on unsatisfied FP/BP dependencies (Section 2.1,
Section 2.2.1).  The three bubble types of Section 2.2.1 (A: epoch start/end, all stages but the first;
B: the wait for the first BP after the warm-up FPs, all but the last; C: unaligned FP/BP inside the epoch,
all but the last) are what this simulation produces; `classify` labels them.

Model: p stages, m micro-batches, every FP takes f and every BP takes b on every stage, hand-over takes no
time, no optimiser step.  Dependencies: FP(s, j) needs FP(s - 1, j); BP(s, j) needs BP(s + 1, j); on the last
stage BP(p - 1, j) needs FP(p - 1, j).  A stage runs its operations serially in a fixed order:

  GPipe (Huang et al. 2019): all m forwards, then all m backwards.
  1F1B  (the non-interleaved schedule DeepSpeed runs, Figure 1 of the paper): min(p - 1 - s, m) warm-up
         forwards, then forward/backward pairs while forwards remain, then the remaining backwards.

  interleaved 1F1B (Narayanan et al. 2021; one of the bubble-reducing schedules the paper's Section 1 and Section
         2.2.2 refer to): every stage (device) holds v model chunks, chunk c of device s being virtual stage c p + s of
         a pipeline of v p virtual stages; an operation is one chunk's FP or BP of one micro-batch and takes f or b
         (here the per-chunk durations).  m must be a multiple of p.  Device s runs, with n = m v operations of each
         kind: min(n, 2 (p - 1 - s) + (v - 1) p) warm-up forwards, then forward/backward pairs while forwards remain,
         then the remaining backwards; its k-th forward is chunk (k mod p v) div p of micro-batch
         (k div p v) p + k mod p, its k-th backward the same micro-batch of chunk v - 1 - (k mod p v) div p.
         Its bubbles add up to (p - 1)(f + b) per device, 1 / v of the plain schedule's for the same model, in more
         and shorter windows.  (v = 1 is a 1F1B schedule with twice the plain one's warm-up forwards.)

An operation starts at max(stage free, dependency finished).  The epoch ends when the last operation anywhere
ends; a stage's bubbles are its maximal idle intervals in [0, epoch end], lead-in and tail included.
All times are integers (nanoseconds by convention) and nothing here is floating point.
"""
from dataclasses import dataclass
from typing import List, Tuple


@dataclass(frozen=True)
class Op:
    kind: str     # "F" or "B"
    mb: int       # micro-batch index
    start: int
    end: int
    chunk: int = 0    # model chunk (interleaved schedule only)


def stage_order(schedule: str, p: int, m: int, s: int) -> List[Tuple[str, int]]:
    """The serial operation order of stage s."""
    if schedule == "gpipe":
        return [("F", j) for j in range(m)] + [("B", j) for j in range(m)]
    if schedule == "1f1b":
        w = min(p - 1 - s, m)
        order = [("F", j) for j in range(w)]
        nf, nb = w, 0
        while nf < m:
            order.append(("F", nf)); nf += 1
            order.append(("B", nb)); nb += 1
        while nb < m:
            order.append(("B", nb)); nb += 1
        return order
    raise ValueError("unknown schedule %r" % schedule)


def simulate(schedule: str, p: int, m: int, f: int, b: int) -> Tuple[List[List[Op]], int]:
    """Timed operations of every stage and the epoch end time."""
    if p < 1 or m < 1 or f <= 0 or b <= 0:
        raise ValueError("p, m >= 1 and f, b > 0 required")
    orders = [stage_order(schedule, p, m, s) for s in range(p)]
    nxt = [0] * p                       # next operation of each stage
    free = [0] * p                      # time each stage becomes free
    done = {}                           # (kind, stage, mb) -> end time
    timed: List[List[Op]] = [[] for _ in range(p)]
    remaining = sum(len(o) for o in orders)
    while remaining:
        progressed = False
        for s in range(p):
            while nxt[s] < len(orders[s]):
                kind, j = orders[s][nxt[s]]
                if kind == "F":
                    dep = 0 if s == 0 else done.get(("F", s - 1, j))
                else:
                    dep = done.get(("F", s, j)) if s == p - 1 else done.get(("B", s + 1, j))
                if dep is None:
                    break
                start = max(free[s], dep)
                end = start + (f if kind == "F" else b)
                done[(kind, s, j)] = end
                timed[s].append(Op(kind, j, start, end))
                free[s] = end
                nxt[s] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("schedule deadlocked")
    return timed, max(free)


def bubbles(schedule: str, p: int, m: int, f: int, b: int, s: int) -> Tuple[List[Tuple[int, int]], int]:
    """Bubble windows [(begin, end), ...] of stage s and the epoch end time T."""
    timed, T = simulate(schedule, p, m, f, b)
    out = []
    t = 0
    for op in timed[s]:
        if op.start > t:
            out.append((t, op.start))
        t = op.end
    if T > t:
        out.append((t, T))
    return out, T


def classify(schedule: str, p: int, m: int, f: int, b: int, s: int) -> List[str]:
    """Type label per bubble of stage s, after Section 2.2.1: 'A' for the lead-in and the tail of the epoch,
    'B' for the idle period right before the stage's first BP, 'C' for every other one."""
    timed, T = simulate(schedule, p, m, f, b)
    ops = timed[s]
    first_b = next(i for i, o in enumerate(ops) if o.kind == "B")
    labels = []
    t = 0
    for i, op in enumerate(ops):
        if op.start > t:
            labels.append("A" if i == 0 else ("B" if i == first_b else "C"))
        t = op.end
    if T > t:
        labels.append("A")
    return labels


def interleaved_order(p: int, m: int, v: int, s: int) -> List[Tuple[str, int, int]]:
    """The serial (kind, micro-batch, chunk) order of device s under the interleaved 1F1B schedule."""
    if v < 1 or m % p != 0:
        raise ValueError("v >= 1 and m a multiple of p required")
    n = m * v

    def fwd(k):
        return ("F", (k // (p * v)) * p + k % p, (k % (p * v)) // p)

    def bwd(k):
        return ("B", (k // (p * v)) * p + k % p, v - 1 - (k % (p * v)) // p)
    w = min(n, 2 * (p - 1 - s) + (v - 1) * p)
    order = [fwd(k) for k in range(w)]
    nf, nb = w, 0
    while nf < n:
        order.append(fwd(nf)); nf += 1
        order.append(bwd(nb)); nb += 1
    while nb < n:
        order.append(bwd(nb)); nb += 1
    return order


def simulate_interleaved(p: int, m: int, v: int, f: int, b: int) -> Tuple[List[List[Op]], int]:
    """Timed operations of every device and the epoch end time; f and b are one chunk's FP and BP durations."""
    if p < 1 or m < 1 or f <= 0 or b <= 0:
        raise ValueError("p, m >= 1 and f, b > 0 required")
    orders = [interleaved_order(p, m, v, s) for s in range(p)]
    last = v * p - 1                    # the last virtual stage
    nxt, free = [0] * p, [0] * p
    done = {}                           # (kind, virtual stage, mb) -> end time
    timed: List[List[Op]] = [[] for _ in range(p)]
    remaining = sum(len(o) for o in orders)
    while remaining:
        progressed = False
        for s in range(p):
            while nxt[s] < len(orders[s]):
                kind, j, c = orders[s][nxt[s]]
                vs = c * p + s
                if kind == "F":
                    dep = 0 if vs == 0 else done.get(("F", vs - 1, j))
                else:
                    dep = done.get(("F", vs, j)) if vs == last else done.get(("B", vs + 1, j))
                if dep is None:
                    break
                start = max(free[s], dep)
                end = start + (f if kind == "F" else b)
                done[(kind, vs, j)] = end
                timed[s].append(Op(kind, j, start, end, c))
                free[s] = end
                nxt[s] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("schedule deadlocked")
    return timed, max(free)


def bubbles_interleaved(p: int, m: int, v: int, f: int, b: int, s: int) -> Tuple[List[Tuple[int, int]], int]:
    """Bubble windows of device s under the interleaved schedule and the epoch end time T."""
    timed, T = simulate_interleaved(p, m, v, f, b)
    out, t = [], 0
    for op in timed[s]:
        if op.start > t:
            out.append((t, op.start))
        t = op.end
    if T > t:
        out.append((t, T))
    return out, T
