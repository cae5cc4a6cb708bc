"""CPU-side tests of the C-ABI library: it loads, exports every declared
symbol, and its host logic (schedule generator, statistics, stage map, layout,
sizing, argument checks) agrees with the oracle and the paper's printed facts."""
import ctypes as C
import itertools
import json
import os
import re

import pytest

import paper_2605_29664_amd as amdp
from paper_2605_29664_amd import binding
from oracle import schedule as S
from oracle import stage as OS
import workloads as W


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(os.path.dirname(amdp.__file__), "..", "include", "amdp.h")).read()
    declared = set(re.findall(r"\b(amdp_[a-z_]+)\s*\(", hdr))
    assert declared == set(binding.EXPORTED)
    L = amdp.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_struct_sizes_match_header_layout():
    assert C.sizeof(amdp.amdp_event_t) == 12
    assert C.sizeof(amdp.amdp_param_desc_t) == 40


def _as_tuples(events):
    return [(e.kind, e.pipeline, e.flags, e.mb, e.version) for e in events]


def test_generator_equals_oracle_over_grid():
    n = 0
    for d in range(1, 13):
        for P in range(1, max(1, d // 2) + 1):
            for i in sorted({0, 1, d // 2, d - 1} & set(range(d))):
                for T in sorted({1, 2, P, 2 * P, d, 2 * d + 1, 4 * d}):
                    for M in sorted({0, 1, T, 3 * T + 1, 5 * T - 1}):
                        for n_inj in (1, 2, 3):
                            for pl, pol in itertools.product((0, 1, 2), (0, 1)):
                                mine = amdp.amdp_schedule_generate(d, P, i, T, M, n_inj, pl, pol)
                                ref = S.generate(d, P, i, T, M, n_inj, pl, pol)
                                assert _as_tuples(mine) == [tuple(e) for e in ref], (d, P, i, T, M, n_inj, pl, pol)
                                n += 1
    assert n > 15000


def test_generator_benchmark_configs_and_stats(golden_dir):
    doc = json.load(open(os.path.join(golden_dir, "derived_schedule_stats.json")))
    for c in doc["cases"]:
        ev = amdp.amdp_schedule_generate(c["d"], c["P"], c["i"], c["T"], c["M"])
        st = amdp.amdp_schedule_stats(ev, c["T"])
        ref = S.stats(S.generate(c["d"], c["P"], c["i"], c["T"], c["M"]), c["T"])
        for k in ("max_inflight", "max_inflight_per_pipeline", "max_mismatch", "max_affected_per_window",
                  "max_live_versions"):
            assert st[k] == ref[k] == c.get(k, ref[k]), (c, k)


def test_stats_equal_oracle_on_odd_cases():
    for args in [(16, 4, 8, 4, 64, 3), (4, 1, 0, 1, 24, 2), (8, 4, 0, 3, 40, 2), (5, 2, 4, 7, 30, 2)]:
        for pl, pol in itertools.product((0, 1), (0, 1)):
            ev = amdp.amdp_schedule_generate(*args, pl, pol)
            ref = S.stats(S.generate(*args, pl, pol), args[3])
            st = amdp.amdp_schedule_stats(ev, args[3])
            for k in st:
                assert st[k] == ref[k], (args, pl, pol, k)


def test_lemma_closed_form_through_the_library(golden_dir):
    for d in (1, 2, 5, 8, 16):
        for n in sorted({1, 2, 3, d}):
            for i in range(d):
                ev = amdp.amdp_schedule_generate(d, 1, i, 1, 6 * d + 12, n, amdp.U_EAGER, amdp.BWD_CURRENT)
                tags = {}
                for e in ev:
                    if e.kind == amdp.EV_F:
                        tags[e.mb] = e.version
                    elif e.kind == amdp.EV_B and 2 * d <= e.mb < 5 * d:
                        assert e.version - tags[e.mb] == min(n, d - i) - 1


def test_fig5_examples_through_the_library(golden_dir):
    facts = json.load(open(os.path.join(golden_dir, "paper_schedule_facts.json")))
    f = facts["fig5_threshold8"]
    ev = amdp.amdp_schedule_generate(f["d"], f["pipelines"], 0, f["threshold"], 32, 2, amdp.U_NEXT_BUBBLE,
                                     amdp.BWD_CURRENT)
    tags = {}
    hit = []
    for e in ev:
        if e.kind == amdp.EV_F:
            tags[e.mb] = e.version
        elif e.kind == amdp.EV_B and f["window"][0] <= e.mb <= f["window"][1] and e.version != tags[e.mb]:
            hit.append(e.mb)
    assert hit == f["mismatched_in_window"]


def test_stage_map_paper_example(golden_dir):
    facts = json.load(open(os.path.join(golden_dir, "paper_schedule_facts.json")))["stage_map_d8"]
    assert [amdp.amdp_stage_map(8, 0, i) for i in range(8)] == facts["pipeline0"]
    assert [amdp.amdp_stage_map(8, 1, i) for i in range(8)] == facts["pipeline1"]
    # every pipeline visits every GPU exactly once
    for d in (2, 4, 6, 8, 16):
        for j in range(d // 2):
            assert sorted(amdp.amdp_stage_map(d, j, i) for i in range(d)) == list(range(d))
    with pytest.raises(amdp.AmdpError):
        amdp.amdp_stage_map(8, 4, 0)


def _cfg(w, **kw):
    args = dict(block_kind=w.block_kind, n_layers=w.n_layers, d_model=w.d_model, n_heads=w.n_heads,
                d_ffn=w.d_ffn, seq_len=w.seq_len, microbatch=w.microbatch, dtype=w.dtype,
                has_lm_head=w.has_lm_head, vocab=w.vocab, ln_eps=w.ln_eps, act_slots=w.act_slots,
                stash_slots=w.stash_slots)
    args.update(kw)
    return binding.make_config(**args)


def test_param_layout_equals_oracle_layout():
    for w in list(W.CONFIGS.values()) + list(W.TINY.values()):
        cfg = _cfg(w)
        mine = amdp.amdp_stage_param_layout(cfg)
        ref = OS.param_layout(w.n_layers, w.d_model, w.d_ffn, w.has_lm_head, w.vocab)
        assert mine == [tuple(r) for r in ref]
        assert amdp.amdp_stage_n_params(cfg) == OS.n_params(ref)


def test_benchmark_parameter_counts():
    want = {1: 198272, 2: 50384896, 3: 75577344, 4: 304363520, 5: 805519360}
    for k, n in want.items():
        assert amdp.amdp_stage_n_params(_cfg(W.CONFIGS[k])) == n


def test_workspace_fits_one_gpu():
    for k, w in W.CONFIGS.items():
        b = amdp.amdp_stage_workspace_bytes(_cfg(w))
        assert 0 < b < 200 * 2 ** 30, (k, b)


def test_bad_configs_are_rejected():
    w = W.CONFIGS[1]
    for kw in (dict(n_heads=3), dict(act_slots=0), dict(stash_slots=0), dict(d_model=0), dict(dtype=7),
               dict(block_kind=5), dict(has_lm_head=True, vocab=0), dict(ln_eps=0.0), dict(seq_len=63)):
        assert amdp.amdp_stage_workspace_bytes(_cfg(w, **kw)) == 0, kw
    bad = _cfg(w)
    bad.struct_size = 8
    assert amdp.amdp_stage_n_params(bad) == 0


def test_generate_rejects_bad_parameters_and_sizes_output():
    with pytest.raises(amdp.AmdpError):
        amdp.amdp_schedule_generate(4, 2, 4, 4, 8)
    with pytest.raises(amdp.AmdpError):
        amdp.amdp_schedule_generate(4, 0, 0, 4, 8)
    assert len(amdp.amdp_schedule_generate(4, 2, 0, 4, 0)) == 0
    p = amdp.amdp_sched_params_t(C.sizeof(amdp.amdp_sched_params_t), 4, 2, 0, 2, 4, 8, 0, 0)
    n = C.c_size_t(0)
    small = (amdp.amdp_event_t * 3)()
    assert amdp.lib().amdp_schedule_generate(C.byref(p), small, 3, C.byref(n)) == amdp.E_CAPACITY
    assert n.value == 3 * 8 + 2
    assert amdp.amdp_strerror(amdp.E_STASH_FULL).startswith("no free weight-version slot")


def test_system_simulation_equals_oracle():
    """The library's timed whole-system simulation reproduces the oracle's
    timeline operation by operation (integer work: exact)."""
    import random
    from oracle import system as OS
    rng = random.Random(2966)
    cases = [(4, 2, 6, 1, 2, 2, 0), (8, 4, 20, 1, 2, 2, 2), (16, 8, 5, 2, 3, 2, 1), (1, 1, 3, 1, 1, 1, 0), (6, 3, 0, 1, 2, 2, 0)]
    for _ in range(40):
        d = rng.randint(1, 10)
        cases.append((d, rng.randint(1, max(1, d // 2)), rng.randint(0, 9), rng.randint(1, 4), rng.randint(1, 7),
                      rng.randint(1, 3), rng.randint(0, 3)))
    for d, P, M, tF, tB, n, pre in cases:
        ops, info = amdp.amdp_system_simulate(d, P, M, tF, tB, n, pre)
        ref_ops, ref = OS.simulate(d, P, M, tF, tB, inject_limit=n, preload=pre)
        assert ops == [tuple(o) for o in ref_ops], (d, P, M, tF, tB, n, pre)
        assert info["makespan"] == ref["makespan"] and info["busy"] == ref["busy"]
        assert info["max_inflight"] == ref["max_inflight"]
        assert info["busy_total"] == sum(ref["busy"]) and info["busy_min"] == min(ref["busy"])
        assert info["busy_max"] == max(ref["busy"])


def test_system_simulation_rejects_bad_parameters():
    for bad in [(0, 1, 1, 1, 1, 2, 0), (4, 3, 1, 1, 1, 2, 0), (4, 2, -1, 1, 1, 2, 0), (4, 2, 1, 0, 1, 2, 0),
                (4, 2, 1, 1, 0, 2, 0), (4, 2, 1, 1, 1, 0, 0), (4, 2, 1, 1, 1, 2, -1)]:
        with pytest.raises(amdp.AmdpError):
            amdp.amdp_system_simulate(*bad)


def test_comparison_schedule_presets():
    """amdp_schedule_preset fills the generator settings of the schedules that
    Table 1 compares; the events equal the oracle's for those settings and
    show the table's weight-version counts."""
    for d in (2, 4, 8):
        M = 6 * d
        for i in range(d):
            ev, p = amdp.amdp_schedule_preset(amdp.PRESET_PIPEDREAM, d, i, M)
            assert (p.pipelines, p.inject_limit, p.threshold, p.update_placement, p.bwd_version) == (1, d, 1, 1, 0)
            assert _as_tuples(ev) == [tuple(e) for e in S.generate(d, 1, i, 1, M, d, S.EAGER, S.STASHED)]
            assert amdp.amdp_schedule_stats(ev, 1)["max_live_versions"] == d - i
            ev, p = amdp.amdp_schedule_preset(amdp.PRESET_PIPEDREAM_2BW, d, i, M)
            assert _as_tuples(ev) == [tuple(e) for e in S.generate(d, 1, i, d, M, d, S.EAGER, S.STASHED)]
            assert amdp.amdp_schedule_stats(ev, d)["max_live_versions"] <= 2
            ev, p = amdp.amdp_schedule_preset(amdp.PRESET_SYNC_1F1B, d, i, M, microbatches=2 * d)
            assert _as_tuples(ev) == [tuple(e) for e in S.generate(d, 1, i, 2 * d, M, d, S.FLUSH, S.STASHED)]
            st = amdp.amdp_schedule_stats(ev, 2 * d)
            assert st["max_mismatch"] == 0 and st["max_live_versions"] == 1
            ev, p = amdp.amdp_schedule_preset(amdp.PRESET_AMDP, d, i, M)
            assert (p.pipelines, p.inject_limit, p.threshold) == (max(1, d // 2), 2, 2 * d)
            assert _as_tuples(ev) == [tuple(e) for e in S.generate(d, max(1, d // 2), i, 2 * d, M, 2, S.NEXT_BUBBLE, S.CURRENT)]
            assert amdp.amdp_schedule_stats(ev, 2 * d)["max_mismatch"] <= 1
    with pytest.raises(amdp.AmdpError):
        amdp.amdp_schedule_preset(amdp.PRESET_SYNC_1F1B, 4, 0, 8)          # needs the microbatch count
    with pytest.raises(amdp.AmdpError):
        amdp.amdp_schedule_preset(7, 4, 0, 8)
