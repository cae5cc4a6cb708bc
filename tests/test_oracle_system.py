"""Pins for the oracle's timed whole-system simulation (oracle/system.py):
closed forms, the paper's statements (Section 3.2), the causal constraints of
Appendix B.4 on random cases, and an independent clock-tick simulation written
here on tiny inputs."""
import itertools
import random

import pytest

from oracle import system as S


def test_stage_map_example_of_section_3_2():
    # d = 8: pipeline 0 walks the GPUs in order, pipeline 1 visits 3,2,1,0,7,6,5,4
    assert [S.stage_map(8, 0, i) for i in range(8)] == [0, 1, 2, 3, 4, 5, 6, 7]
    assert [S.stage_map(8, 1, i) for i in range(8)] == [3, 2, 1, 0, 7, 6, 5, 4]
    # every pipeline visits every GPU once, so each GPU hosts one stage of each pipeline
    for d in (2, 4, 6, 8, 16):
        for j in range(max(1, d // 2)):
            assert sorted(S.stage_map(d, j, i) for i in range(d)) == list(range(d))


@pytest.mark.parametrize("d,tF,tB,M", [(1, 1, 1, 3), (4, 1, 2, 5), (5, 3, 7, 4), (8, 2, 2, 3)])
def test_one_minibatch_at_a_time_closed_form(d, tF, tB, M):
    """n = 1: the pipeline is serial. Minibatch m starts at m*d*(tF+tB); its
    forward of stage i starts i*tF later, its backward of stage i after the d
    forwards and the d-1-i backwards above it. Every GPU is busy 1/d of the time."""
    ops, info = S.simulate(d, 1, M, tF, tB, inject_limit=1)
    assert info["makespan"] == M * d * (tF + tB)
    assert info["busy"] == [M * (tF + tB)] * d
    start = {(o.kind, o.stage, o.mb): o.start for o in ops}
    for m in range(M):
        base = m * d * (tF + tB)
        for i in range(d):
            assert start[(S.F, i, m)] == base + i * tF
            assert start[(S.B, i, m)] == base + d * tF + (d - 1 - i) * tB
            assert S.stage_map(d, 0, i) == i


@pytest.mark.parametrize("d,n,tF,tB", [(4, 2, 1, 2), (8, 2, 1, 2), (8, 2, 1, 1), (8, 3, 2, 3), (16, 2, 1, 2)])
def test_active_ratio_is_n_over_d(d, n, tF, tB):
    """Section 3.2: with n minibatches in flight one pipeline keeps a GPU busy
    n/d of the time (n = 1: 1/d, n = 2: 2/d)."""
    M = 400
    ops, info = S.simulate(d, 1, M, tF, tB, inject_limit=n)
    for b in info["busy"]:
        assert abs(b / info["makespan"] - n / d) < 0.01 * n / d
    assert info["max_inflight"] == n


@pytest.mark.parametrize("d,tF,tB", [(4, 1, 2), (8, 1, 2), (4, 1, 1), (8, 2, 4)])
def test_half_depth_pipelines_with_preloading_leave_no_bubbles(d, tF, tB):
    """Section 3.2: d/2 pipelines, and floor(t_B / t_F) preloaded minibatches
    (at least the two a forward-backward pair needs at d = 8 with equal costs),
    fill the machine when backward costs once or twice a forward; with the
    strict limit of two the bubbles are large. (Other cost ratios keep the
    "middle bubble" the section says cannot be removed.)"""
    M = 300
    pre = max(tB // tF, 2 if d > 4 else 1)
    _, full = S.simulate(d, d // 2, M, tF, tB, preload=pre)
    _, strict = S.simulate(d, d // 2, M, tF, tB, preload=0)
    util = lambda info: sum(info["busy"]) / (d * info["makespan"])
    assert util(full) > 0.99
    assert util(strict) < 0.85
    assert sum(full["busy"]) == sum(strict["busy"]) == (d // 2) * M * d * (tF + tB)


def _check_constraints(d, P, M, tF, tB, n, pre, ops):
    assert len(ops) == 2 * d * P * M
    by = {(o.pipeline, o.kind, o.stage, o.mb): o for o in ops}
    assert len(by) == len(ops)
    for o in ops:
        assert o.end - o.start == (tF if o.kind == S.F else tB)
        assert o.gpu == S.stage_map(d, o.pipeline, o.stage)
    for j in range(P):
        for m in range(M):
            for i in range(d):
                f, b = by[(j, S.F, i, m)], by[(j, S.B, i, m)]
                assert f.end <= b.start                                   # forward before backward
                if i + 1 < d:
                    assert f.end <= by[(j, S.F, i + 1, m)].start          # forward chain
                    assert by[(j, S.B, i + 1, m)].end <= b.start          # backward chain
                if m + 1 < M:
                    assert f.start < by[(j, S.F, i, m + 1)].start         # minibatch order kept per stage
                    assert b.start < by[(j, S.B, i, m + 1)].start
            if m >= n + pre:                                              # injection limit at stage 0
                assert by[(j, S.F, 0, m)].start >= by[(j, S.B, 0, m - n - pre)].end
    for g in range(d):                                                    # one operation at a time
        mine = sorted((o.start, o.end) for o in ops if o.gpu == g)
        for (s0, e0), (s1, e1) in zip(mine, mine[1:]):
            assert e0 <= s1


def test_causal_constraints_on_random_cases():
    rng = random.Random(29664)
    for _ in range(60):
        d = rng.randint(1, 9)
        P = rng.randint(1, max(1, d // 2))
        M, tF, tB = rng.randint(0, 7), rng.randint(1, 4), rng.randint(1, 6)
        n, pre = rng.randint(1, 3), rng.randint(0, 2)
        ops, info = S.simulate(d, P, M, tF, tB, inject_limit=n, preload=pre)
        _check_constraints(d, P, M, tF, tB, n, pre, ops)
        assert info["max_inflight"] <= n + pre
        assert sum(info["busy"]) == P * M * d * (tF + tB)
        assert info["makespan"] == max([o.end for o in ops], default=0)


def _tick_simulation(d, P, M, tF, tB, n, pre):
    """The same rules, advanced one time unit at a time with plain lists."""
    limit = n + pre
    ready = [[] for _ in range(d)]          # (ready_time, kind, pipeline, mb, stage)
    running = [None] * d
    out = []
    nxt = [min(limit, M)] * P
    for j in range(P):
        for m in range(min(limit, M)):
            ready[S.stage_map(d, j, 0)].append((0, S.F, j, m, 0))
    t, left = 0, 2 * d * P * M
    while left:
        for g in range(d):
            r = running[g]
            if r is not None and r[-1] == t:
                kind, j, i, m, s, e = r
                running[g] = None
                out.append((kind, j, i, m, g, s, e))
                left -= 1
                if kind == S.F:
                    nk, ni = (S.F, i + 1) if i + 1 < d else (S.B, i)
                    ready[S.stage_map(d, j, ni)].append((t, nk, j, m, ni))
                elif i > 0:
                    ready[S.stage_map(d, j, i - 1)].append((t, S.B, j, m, i - 1))
                elif nxt[j] < M:
                    ready[S.stage_map(d, j, 0)].append((t, S.F, j, nxt[j], 0))
                    nxt[j] += 1
        for g in range(d):
            if running[g] is None and ready[g]:
                best = min(ready[g], key=lambda r: (r[0], -r[1], r[2], r[3], r[4]))
                ready[g].remove(best)
                _, kind, j, m, i = best
                running[g] = (kind, j, i, m, t, t + (tF if kind == S.F else tB))
        t += 1
    return sorted(out, key=lambda o: (o[5], o[4]))


@pytest.mark.parametrize("d,P,M,tF,tB,n,pre", [(4, 2, 4, 1, 2, 2, 0), (4, 2, 5, 1, 2, 2, 2), (6, 3, 3, 2, 3, 2, 1),
                                               (3, 1, 4, 1, 1, 2, 0), (8, 4, 3, 1, 2, 2, 2), (2, 1, 3, 2, 1, 1, 0)])
def test_event_driven_equals_clock_tick_simulation(d, P, M, tF, tB, n, pre):
    ops, _ = S.simulate(d, P, M, tF, tB, inject_limit=n, preload=pre)
    assert [tuple(o) for o in ops] == _tick_simulation(d, P, M, tF, tB, n, pre)


def test_conflicting_backwards_are_served_in_order_of_arrival():
    """Two counter-directed pipelines on four GPUs (the paper's Figure 3 setting):
    whenever two operations wait for one GPU, the one that was ready first runs
    first, and at equal ready times a backward goes before a forward."""
    ops, _ = S.simulate(4, 2, 6, 1, 2)
    ready_time = {}
    by = {(o.pipeline, o.kind, o.stage, o.mb): o for o in ops}
    for o in ops:
        if o.kind == S.F:
            rt = by[(o.pipeline, S.F, o.stage - 1, o.mb)].end if o.stage else (
                0 if o.mb < 2 else by[(o.pipeline, S.B, 0, o.mb - 2)].end)
        else:
            rt = by[(o.pipeline, S.F, 3, o.mb)].end if o.stage == 3 else by[(o.pipeline, S.B, o.stage + 1, o.mb)].end
        ready_time[o] = rt
    waited = 0
    for g in range(4):
        mine = sorted((o for o in ops if o.gpu == g), key=lambda o: o.start)
        for a, b in itertools.combinations(mine, 2):       # a starts before b
            if ready_time[b] < a.start:                    # b was already waiting when a started
                assert (ready_time[a], -a.kind) <= (ready_time[b], -b.kind)
                waited += 1
    assert waited > 0          # the case does contain conflicts


@pytest.mark.parametrize("d,n,tF,tB", [(4, 4, 1, 2), (8, 8, 1, 2), (6, 3, 1, 2), (8, 5, 2, 3), (2, 2, 1, 1)])
def test_one_flushed_minibatch_has_the_bubble_ratio_of_table_1(d, n, tF, tB):
    """One pipeline, one minibatch of n <= d microbatches all admitted at once
    and then drained: the classic synchronous schedule, whose bubble ratio
    Table 1 prints as (d-1)/(n+d-1)."""
    _, info = S.simulate(d, 1, n, tF, tB, inject_limit=d)
    assert info["makespan"] == (n + d - 1) * (tF + tB)
    bubble = 1 - sum(info["busy"]) / (d * info["makespan"])
    assert abs(bubble - (d - 1) / (n + d - 1)) < 1e-12
