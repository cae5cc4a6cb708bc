"""Oracle: the per-stage AMDP event order and its weight-version tags.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What the paper fixes (Sections 3.1-3.3, Lemma 1, Appendix B.4):
  * a stage alternates one forward and one backward (1F1B) after a warm-up in
    which stage i of a depth-d pipeline reads w = min(n, d - i) minibatches,
    n being the number stage 0 may inject before its first backward
    (Section 3.1); AMDP sets n = 2;
  * several pipelines run concurrently on distinct minibatches and the
    replicas of one stage pool their gradients (Section 3.2);
  * gradients are summed over a window of T minibatches and applied in one
    update "during the next bubble" (Section 3.3);
  * the parameter mismatch of a minibatch is the number of updates that fall
    between its forward and its backward at this stage (Section 3.1);
  * forward precedes backward for each minibatch and minibatch order is kept
    at every stage (Appendix B.4).

What the paper leaves open, and the reading taken here (all listed in the
design notes of this repository):
  * minibatch m belongs to pipeline m mod P and window m div T;
  * the P replicas of the stage are merged round by round onto one logical
    stage: a forward round is one forward per pipeline, a backward round one
    backward per pipeline, each backward followed at once by the accumulation
    of its gradient;
  * a third placement, "flush", gives the synchronous comparison schedule of
    Table 1 (1F1B with a pipeline flush): a window's minibatches are drained
    and its update applied before the next window's first forward;
  * "next bubble" placement: the update closing window u is applied
    immediately before the first backward of window u+1 (this is the only
    placement that reproduces both statements made about Figure 5); the
    "eager" placement applies it right after the window's last accumulation,
    which is the setting Lemma 1 describes;
  * backward either reuses the forward's version (a stash) or takes whatever
    is current (the mismatch the paper counts).
"""
from collections import namedtuple

F, B, A, U = 0, 1, 2, 3
KIND_NAMES = "FBAU"

NEXT_BUBBLE, EAGER, FLUSH = 0, 1, 2
STASHED, CURRENT = 0, 1

FLAG_LAST_USE = 1       # last forward/backward that reads this version
FLAG_PARTIAL_WINDOW = 2  # update closes a window with fewer than T minibatches

Event = namedtuple("Event", "kind pipeline flags mb version")


def generate(depth, pipelines, stage, threshold, n_minibatches, inject_limit=2,
             placement=NEXT_BUBBLE, bwd_version=STASHED):
    """Ordered events of one logical stage.

    F/B/A events carry the global minibatch id in `mb`; U events carry the
    window index. `version` is the weight version a forward/backward reads
    (the number of updates applied before it, or the forward's tag under the
    stash policy), 0 for A, and the version produced for U.
    """
    d, P, i, T, M, n = depth, pipelines, stage, threshold, n_minibatches, inject_limit
    if not (d >= 1 and P >= 1 and 0 <= i < d and T >= 1 and M >= 0 and n >= 1):
        raise ValueError("bad schedule parameters")
    w = min(n, d - i)                      # warm-up forwards per pipeline, Section 3.1
    def one_f_one_b(first, last):
        """1F1B per replica over minibatches [first, last): w forward rounds,
        then backward round g / forward round g+w."""
        n_rounds = -(-(last - first) // P) if last > first else 0      # ceil
        fwd_round = lambda g: [(F, m) for m in range(first + g * P, min(first + (g + 1) * P, last))]

        def bwd_round(g):
            out = []
            for m in range(first + g * P, min(first + (g + 1) * P, last)):
                out += [(B, m), (A, m)]
            return out
        out = []
        for g in range(min(w, n_rounds)):
            out += fwd_round(g)
        for g in range(n_rounds):
            out += bwd_round(g)
            if g + w < n_rounds:
                out += fwd_round(g + w)
        return out

    if placement == FLUSH:
        # synchronous schedule: a window is drained and its update applied before
        # any forward of the next window (the classic 1F1B with a flush)
        order = []
        for first in range(0, M, T):
            order += one_f_one_b(first, min(first + T, M))
    else:
        order = one_f_one_b(0, M)

    # place the updates
    n_updates = -(-M // T) if M else 0
    seq = []
    for kind, m in order:
        if placement == NEXT_BUBBLE and kind == B and m % T == 0 and m > 0:
            seq.append((U, m // T - 1))
        seq.append((kind, m))
        if placement in (EAGER, FLUSH) and kind == A and ((m + 1) % T == 0 or (placement == FLUSH and m == M - 1)):
            seq.append((U, m // T))
    placed = sum(1 for k, _ in seq if k == U)
    for u in range(placed, n_updates):     # the last (possibly short) window
        seq.append((U, u))

    # version tags
    events = []
    applied = 0
    fwd_tag = {}
    for kind, m in seq:
        if kind == F:
            fwd_tag[m] = applied
            events.append([F, m % P, 0, m, applied])
        elif kind == B:
            tag = fwd_tag[m] if bwd_version == STASHED else applied
            events.append([B, m % P, 0, m, tag])
        elif kind == A:
            events.append([A, m % P, 0, m, 0])
        else:
            applied += 1
            short = (m + 1) * T > M
            events.append([U, 0, FLAG_PARTIAL_WINDOW if short else 0, m, applied])

    # mark the last reader of every version
    seen = set()
    for ev in reversed(events):
        if ev[0] in (F, B) and ev[4] not in seen:
            seen.add(ev[4])
            ev[2] |= FLAG_LAST_USE
    return [Event(*ev) for ev in events]


def mismatch_per_minibatch(events):
    """Updates strictly between F(m) and B(m), for every m (Section 3.1)."""
    applied = 0
    at_f = {}
    out = {}
    for ev in events:
        if ev.kind == U:
            applied += 1
        elif ev.kind == F:
            at_f[ev.mb] = applied
        elif ev.kind == B:
            out[ev.mb] = applied - at_f[ev.mb]
    return out


def stats(events, threshold=None):
    """Bounds a schedule must respect: in-flight minibatches (forward done,
    backward not started) merged and per pipeline, the largest mismatch, the
    number of mismatched minibatches per window, and how many weight versions
    must be resident at once (the current one plus every older one a later
    event still reads)."""
    inflight = set()
    per_pipe = {}
    max_inflight = 0
    max_pp = 0
    for ev in events:
        if ev.kind == F:
            inflight.add(ev.mb)
            per_pipe[ev.pipeline] = per_pipe.get(ev.pipeline, 0) + 1
        elif ev.kind == B:
            inflight.discard(ev.mb)
            per_pipe[ev.pipeline] -= 1
        max_inflight = max(max_inflight, len(inflight))
        max_pp = max(max_pp, max(per_pipe.values(), default=0))

    mm = mismatch_per_minibatch(events)
    affected = {}
    if threshold:
        for m, k in mm.items():
            if k > 0:
                affected[m // threshold] = affected.get(m // threshold, 0) + 1

    # residency: walk backwards collecting versions still to be read
    future = [None] * len(events)
    need = {}
    for idx in range(len(events) - 1, -1, -1):
        ev = events[idx]
        if ev.kind in (F, B):
            need[ev.version] = need.get(ev.version, 0) + 1
        future[idx] = set(need)
    applied = 0
    max_live = 1
    for idx, ev in enumerate(events):
        if ev.kind == U:
            applied += 1
        live = {v for v in future[idx] if v <= applied} | {applied}
        max_live = max(max_live, len(live))
    return {
        "max_inflight": max_inflight,
        "max_inflight_per_pipeline": max_pp,
        "max_mismatch": max(mm.values(), default=0),
        "max_affected_per_window": max(affected.values(), default=0),
        "max_live_versions": max_live,
        "mismatched": sorted(m for m, k in mm.items() if k > 0),
    }


def render(events):
    """Compact text form, e.g. 'F0[0] F1[0] B0[0] A0 U0>1'."""
    parts = []
    for ev in events:
        k = KIND_NAMES[ev.kind]
        if ev.kind == A:
            parts.append(f"A{ev.mb}")
        elif ev.kind == U:
            parts.append(f"U{ev.mb}>{ev.version}")
        else:
            parts.append(f"{k}{ev.mb}[{ev.version}]")
    return " ".join(parts)
