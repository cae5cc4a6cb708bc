"""Pins for oracle/schedule.py against what the paper prints and against
brute force (no GPU)."""
import itertools
import json
import os

import pytest

from oracle import schedule as S


@pytest.fixture(scope="module")
def facts(golden_dir):
    return json.load(open(os.path.join(golden_dir, "paper_schedule_facts.json")))


def steady(mm, lo, hi):
    return {mm[m] for m in range(lo, hi)}


# --- Lemma 1 / Lemma B.1: mismatch(i) = min(n, d-i) - 1 ----------------------
# Setting of the lemma: one pipeline, an update right after every backward.
@pytest.mark.parametrize("d", range(1, 17))
def test_lemma_closed_form(d):
    for n in sorted({1, 2, 3, d}):
        for i in range(d):
            ev = S.generate(d, 1, i, 1, 6 * d + 12, inject_limit=n, placement=S.EAGER,
                            bwd_version=S.CURRENT)
            mm = S.mismatch_per_minibatch(ev)
            assert steady(mm, 2 * d, 5 * d) == {min(n, d - i) - 1}, (d, n, i)
            # the tag difference a CURRENT-policy backward sees is that same number
            tags = {}
            for e in ev:
                if e.kind == S.F:
                    tags[e.mb] = e.version
                elif e.kind == S.B and 2 * d <= e.mb < 5 * d:
                    assert e.version - tags[e.mb] == min(n, d - i) - 1


def test_lemma_printed_special_cases(facts):
    for c in facts["lemma_special_cases"]["cases"]:
        ev = S.generate(c["d"], 1, c["stage"], 1, 40, inject_limit=c["n"], placement=S.EAGER)
        assert steady(S.mismatch_per_minibatch(ev), 10, 30) == {c["mismatch"]}


@pytest.mark.parametrize("d", [2, 4, 8, 16, 31])
def test_amdp_bound_n2(d):
    for i in range(d):
        ev = S.generate(d, 1, i, 1, 80, inject_limit=2, placement=S.EAGER)
        assert max(S.mismatch_per_minibatch(ev).values()) <= 1


# --- Section 3.3 / Figure 5 worked examples ---------------------------------
def test_fig5_threshold_8(facts):
    f = facts["fig5_threshold8"]
    for i in range(f["d"] - 1):     # every stage that warms up with two forwards
        ev = S.generate(f["d"], f["pipelines"], i, f["threshold"], 32)
        mm = S.mismatch_per_minibatch(ev)
        lo, hi = f["window"]
        hit = [m for m in range(lo, hi + 1) if mm[m] > 0]
        assert hit == f["mismatched_in_window"]
        assert all(mm[m] == 1 for m in hit)


def test_fig5_threshold_4(facts):
    f = facts["fig5_threshold4"]
    ev = S.generate(f["d"], f["pipelines"], 0, f["threshold"], 32)
    mm = S.mismatch_per_minibatch(ev)
    # every minibatch after the first window (the first update has not happened before it)
    assert {mm[m] for m in range(f["threshold"], 28)} == {f["every_minibatch_mismatch"]}


def test_hazard_without_accumulation(facts):
    # one pipeline, update per minibatch, update deferred to the next bubble:
    # two updates land between a forward and its backward (Section 3.3)
    ev = S.generate(4, 1, 0, 1, 24, placement=S.NEXT_BUBBLE)
    assert S.stats(ev, 1)["max_mismatch"] == facts["unaccumulated_hazard"]["mismatch"]


def test_worked_example_text():
    ev = S.generate(4, 2, 0, 8, 16)
    txt = S.render(ev)
    assert txt.startswith("F0[0] F1[0] F2[0] F3[0] B0[0] A0 B1[0] A1 F4[0] F5[0] B2[0] A2 B3[0] A3")
    assert "F10[0] F11[0] U0>1 B8[0] A8 B9[0] A9 F12[1] F13[1]" in txt


# --- whole-pipeline executability (Appendix B.4 causal constraints) ----------
def _pipeline_executes(d, n, M):
    """Run the per-stage orders of all d stages of ONE pipeline together under
    F(i,j) < F(i+1,j), B(i+1,j) < B(i,j), F(i,j) < B(i,j). Returns the
    largest number of minibatches stage 0 had in flight, or None on deadlock."""
    orders = []
    for i in range(d):
        ev = S.generate(d, 1, i, 1, M, inject_limit=n, placement=S.EAGER)
        orders.append([(e.kind, e.mb) for e in ev if e.kind in (S.F, S.B)])
    pos = [0] * d
    done = set()
    inflight0 = 0
    worst = 0
    progressed = True
    while progressed:
        progressed = False
        for i in range(d):
            while pos[i] < len(orders[i]):
                kind, m = orders[i][pos[i]]
                if kind == S.F:
                    ready = i == 0 or (S.F, i - 1, m) in done
                else:
                    ready = (S.F, i, m) in done and (i == d - 1 or (S.B, i + 1, m) in done)
                if not ready:
                    break
                done.add((kind, i, m))
                pos[i] += 1
                progressed = True
                if i == 0:
                    inflight0 += 1 if kind == S.F else -1
                    worst = max(worst, inflight0)
    if any(pos[i] < len(orders[i]) for i in range(d)):
        return None
    return worst


@pytest.mark.parametrize("d", [1, 2, 3, 4, 6, 8, 12])
def test_all_stages_execute_together(d):
    for n in sorted({1, 2, 3, d}):
        worst = _pipeline_executes(d, n, 3 * d + 5)
        assert worst is not None, "per-stage orders deadlock"
        assert worst == min(n, d)            # stage 0 injects exactly its limit, never more


# --- brute-force invariants of the merged multi-pipeline order ----------------
def _check_invariants(d, P, i, T, M, placement, policy):
    ev = S.generate(d, P, i, T, M, placement=placement, bwd_version=policy)
    w = min(2, d - i)
    n_u = -(-M // T)
    assert len(ev) == 3 * M + n_u
    seen_f, seen_b, seen_a = set(), set(), set()
    last_b = {}
    inflight = {}
    applied = 0
    resident = {0}
    for idx, e in enumerate(ev):
        if e.kind == S.F:
            assert e.mb not in seen_f and e.pipeline == e.mb % P
            assert e.version == applied
            seen_f.add(e.mb)
            inflight[e.pipeline] = inflight.get(e.pipeline, 0) + 1
            assert inflight[e.pipeline] <= w
        elif e.kind == S.B:
            assert e.mb in seen_f and e.mb not in seen_b
            assert last_b.get(e.pipeline, -1) < e.mb            # FIFO per replica
            last_b[e.pipeline] = e.mb
            seen_b.add(e.mb)
            inflight[e.pipeline] -= 1
            assert e.version in resident, "backward reads a version that was dropped"
            # an update of window u lies before any backward of window u+2
            assert applied >= e.mb // T - 1
        elif e.kind == S.A:
            assert ev[idx - 1].kind == S.B and ev[idx - 1].mb == e.mb
            seen_a.add(e.mb)
        else:
            applied += 1
            assert e.version == applied and e.mb == applied - 1
            upto = min((e.mb + 1) * T, M)
            assert all(m in seen_a for m in range(e.mb * T, upto)), "update before its window closed"
            assert not any(m in seen_a for m in range(upto, M)), "update after next window's accumulation"
            resident.add(applied)
        if e.kind in (S.F, S.B) and e.flags & S.FLAG_LAST_USE and e.version != applied:
            resident.discard(e.version)
    assert seen_f == seen_b == seen_a == set(range(M)) and applied == n_u
    st = S.stats(ev, T)
    bound = -(-(w * P) // T) if placement == S.NEXT_BUBBLE else -(-(w * P - 1) // T)
    assert st["max_mismatch"] <= bound
    if T >= 2 * P:
        assert st["max_mismatch"] <= 1
    if P <= max(1, d // 2):
        assert st["max_affected_per_window"] <= max(w * P, 1) <= max(d, 2)
    assert st["max_live_versions"] <= 1 + min(w, -(-(w * P) // T)) + (1 if placement == S.NEXT_BUBBLE and T < w * P else 0)
    assert st["max_inflight_per_pipeline"] <= w and st["max_inflight"] <= w * P


def test_invariants_brute_force():
    n = 0
    for d in range(1, 13):
        for P in range(1, max(1, d // 2) + 1):
            for i in sorted({0, 1, d // 2, d - 2, d - 1} & set(range(d))):
                for T in sorted({1, 2, P, 2 * P, d, 2 * d + 1, 4 * d}):
                    for M in sorted({0, 1, T, 3 * T, 3 * T + 1, 5 * T - 1}):
                        for placement, policy in itertools.product((S.NEXT_BUBBLE, S.EAGER),
                                                                   (S.STASHED, S.CURRENT)):
                            _check_invariants(d, P, i, T, M, placement, policy)
                            n += 1
    assert n > 5000


def test_stashed_vs_current_tags():
    ev_s = S.generate(6, 3, 3, 8, 40, bwd_version=S.STASHED)
    ev_c = S.generate(6, 3, 3, 8, 40, bwd_version=S.CURRENT)
    assert [(e.kind, e.mb) for e in ev_s] == [(e.kind, e.mb) for e in ev_c]
    mm = S.mismatch_per_minibatch(ev_s)
    for a, b in zip(ev_s, ev_c):
        if a.kind == S.B:
            assert b.version - a.version == mm[a.mb]
        elif a.kind == S.F:
            assert a.version == b.version


def test_derived_goldens(golden_dir):
    doc = json.load(open(os.path.join(golden_dir, "derived_schedule_stats.json")))
    for c in doc["cases"]:
        st = S.stats(S.generate(c["d"], c["P"], c["i"], c["T"], c["M"]), c["T"])
        for k in ("max_mismatch", "max_inflight", "max_inflight_per_pipeline", "max_live_versions",
                  "mismatched"):
            assert st[k] == c[k], (c, k)


def test_three_stashed_versions_reachable():
    # stress list for a stash of capacity 3: injection limit 3, short windows
    ev = S.generate(16, 4, 8, 4, 64, inject_limit=3)
    st = S.stats(ev, 4)
    assert st["max_live_versions"] == 4 and st["max_mismatch"] == 3


# ---------------------------------------------------------------- comparison schedules of Table 1
@pytest.mark.parametrize("d,T,M", [(4, 4, 12), (4, 6, 15), (8, 8, 16), (6, 3, 7)])
def test_flushed_schedule_is_synchronous(d, T, M):
    """FLUSH placement: every window is a complete 1F1B schedule of its own
    followed by its update, so no minibatch sees an update between its forward
    and backward, one version is live, and the events of window u are exactly
    the events of a stand-alone schedule of its minibatches shifted by u*T."""
    for i in range(d):
        ev = S.generate(d, 1, i, T, M, inject_limit=d, placement=S.FLUSH)
        st = S.stats(ev, T)
        assert st["max_mismatch"] == 0 and st["max_live_versions"] == 1
        assert st["max_inflight"] == min(d - i, T, M)
        assert all(e.version == e.mb // T for e in ev if e.kind in (S.F, S.B))
        pos = 0
        for u in range(-(-M // T)):
            size = min(T, M - u * T)
            alone = S.generate(d, 1, i, size, size, inject_limit=d, placement=S.EAGER)
            chunk = ev[pos:pos + len(alone)]
            assert [(e.kind, e.mb) for e in chunk if e.kind != S.U] == \
                   [(e.kind, e.mb + u * T) for e in alone if e.kind != S.U]
            assert chunk[-1].kind == S.U and chunk[-1].mb == u
            pos += len(alone)
        assert pos == len(ev)


@pytest.mark.parametrize("d", [2, 4, 8])
def test_weight_versions_of_the_asynchronous_comparison_schedules(d):
    """Table 1's weight-memory column: PipeDream keeps between one and d weight
    versions (d - i at stage i: one per minibatch in flight), PipeDream-2BW two,
    AMDP one besides the current (its backward uses the current weights and is
    off by at most one update, Lemma 1)."""
    M = 6 * d
    for i in range(d):
        pd = S.generate(d, 1, i, 1, M, inject_limit=d, placement=S.EAGER, bwd_version=S.STASHED)
        assert S.stats(pd, 1)["max_live_versions"] == d - i
        assert S.stats(pd, 1)["max_mismatch"] == d - i - 1            # what stashing hides from backward
        bw = S.generate(d, 1, i, d, M, inject_limit=d, placement=S.EAGER, bwd_version=S.STASHED)
        assert S.stats(bw, d)["max_live_versions"] == (2 if i < d - 1 else 1)
        am = S.generate(d, max(1, d // 2), i, 2 * d, M, inject_limit=2, placement=S.NEXT_BUBBLE,
                        bwd_version=S.CURRENT)
        assert S.stats(am, 2 * d)["max_mismatch"] <= 1
