"""Oracle: timed simulation of the whole multi-directional pipeline system.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What the paper fixes (Section 3.2, Appendix B.4):
  * d GPUs, P pipelines (P = d/2 removes the bubbles); stage i of pipeline j
    runs on GPU (2j + i) mod d for even j and (2j - i + d + 1) mod d for odd j;
  * pipelines work on distinct minibatches; stage 0 of a pipeline lets at most
    n minibatches be in flight (n = 2), which keeps a GPU busy for a fraction
    r = n/d of the time per pipeline;
  * forward(i, m) precedes forward(i+1, m) and backward(i, m); backward(i, m)
    precedes backward(i-1, m); every stage keeps the order of its minibatches;
  * a GPU asked for two operations at once runs the one that was ready first
    (FIFO) and defers the other;
  * forward and backward cost differently (backward about twice forward).

What it leaves open, and the reading taken here:
  * time is an integer number of units; a forward of any stage takes t_forward,
    a backward t_backward; transfers between GPUs take no time;
  * operations are not preempted; a free GPU starts, among its operations that
    are ready, the one with the earliest ready time; ties go to a backward
    before a forward, then to the lower pipeline, then to the lower minibatch;
  * "preloading" (extra forwards injected at segment boundaries, as many as
    floor(t_B / t_F)) is a parameter `preload`: stage 0 may have n + preload
    minibatches in flight; 0 keeps the strict limit.
"""
import heapq
from collections import namedtuple

F, B = 0, 1
Op = namedtuple("Op", "kind pipeline stage mb gpu start end")


def stage_map(depth, pipeline, stage):
    """GPU that hosts `stage` of `pipeline` (Section 3.2)."""
    d, j, i = depth, pipeline, stage
    return (2 * j + i) % d if j % 2 == 0 else (2 * j - i + d + 1) % d


def simulate(depth, pipelines, minibatches, t_forward=1, t_backward=2, inject_limit=2, preload=0):
    """Runs `minibatches` minibatches through each of `pipelines` pipelines.

    Returns (ops, info): ops in start order (ties: by GPU), info = dict with
    makespan, busy (per GPU), max_inflight (per pipeline, at stage 0).
    """
    d, P, M, tF, tB = depth, pipelines, minibatches, t_forward, t_backward
    if not (d >= 1 and 1 <= P <= max(1, d // 2) and M >= 0 and tF >= 1 and tB >= 1 and inject_limit >= 1
            and preload >= 0):
        raise ValueError("bad simulation parameters")
    limit = inject_limit + preload
    ready = [[] for _ in range(d)]          # per GPU: heap of (ready_time, -kind, pipeline, mb, stage)
    free_at = [0] * d
    busy = [0] * d
    running = [None] * d
    ops = []
    inflight = [0] * P
    max_inflight = 0
    events = []                             # heap of completion times

    def make_ready(t, kind, j, m, i):
        heapq.heappush(ready[stage_map(d, j, i)], (t, -kind, j, m, i))

    for j in range(P):
        for m in range(min(limit, M)):
            make_ready(0, F, j, m, 0)
        inflight[j] = min(limit, M)
        max_inflight = max(max_inflight, inflight[j])
    next_inject = [min(limit, M)] * P

    t = 0
    while True:
        # start whatever can start at time t
        for g in range(d):
            if running[g] is None and ready[g] and ready[g][0][0] <= t:
                rt, nk, j, m, i = heapq.heappop(ready[g])
                kind = -nk
                dur = tF if kind == F else tB
                running[g] = (kind, j, i, m, t, t + dur)
                busy[g] += dur
                heapq.heappush(events, t + dur)
        if not events:
            break
        t = heapq.heappop(events)
        while events and events[0] == t:
            heapq.heappop(events)
        # finish everything that ends at t, GPU by GPU
        for g in range(d):
            r = running[g]
            if r is None or r[5] != t:
                continue
            kind, j, i, m, s, e = r
            running[g] = None
            ops.append(Op(kind, j, i, m, g, s, e))
            if kind == F:
                if i + 1 < d:
                    make_ready(t, F, j, m, i + 1)
                else:
                    make_ready(t, B, j, m, i)
            else:
                if i > 0:
                    make_ready(t, B, j, m, i - 1)
                else:
                    inflight[j] -= 1
                    if next_inject[j] < M:
                        make_ready(t, F, j, next_inject[j], 0)
                        next_inject[j] += 1
                        inflight[j] += 1
                        max_inflight = max(max_inflight, inflight[j])
    ops.sort(key=lambda o: (o.start, o.gpu))
    makespan = max([o.end for o in ops], default=0)
    return ops, dict(makespan=makespan, busy=busy, max_inflight=max_inflight)
