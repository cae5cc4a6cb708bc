"""GPU parity at the benchmark's full sizes, in the launch configuration
bench.py times (default options, the stage's own choice of side stream).

  (a) every configuration at FULL DEPTH: the first minibatch's forward,
      backward (Y or the loss, dX, every parameter's slice of g),
      accumulation and the update, against the fp64 oracle (5 to 40 s of
      oracle time per minibatch on 16 host cores);
  (b) configuration 2 through its whole AMDP schedule: two windows with the
      forward's version in backward (22 minibatches, two updates, one older
      version resident across each update), and one window plus the
      minibatches in flight across the update with the CURRENT version in
      backward (the parameter mismatch of Section 3.1 at full width);
  (c) configuration 5's width with three older weight versions resident beside
      the current one and each of them selected by a backward (one layer);
  (d) the paper-shaped widths and the first stage at one layer; the streaming
      kernels on configuration 5's 805 M parameters, on sampled entries."""
import numpy as np
import pytest

import workloads as W
from oracle import optim
from oracle import schedule as OSched
from tests.parity import run_parity, worst_entries, GpuStage, rel_err, TOL

pytestmark = pytest.mark.gpu


def _show(tag, rep):
    print(f"[{tag}] ok={rep['ok']} worst={rep['worst']:.3e} elem={rep['worst_elem']:.3e} events={rep['events']} "
          f"resident<= {rep['max_resident_versions']} {rep['seconds']:.0f}s", worst_entries(rep, 3), flush=True)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("k", [2, 3, 4, 5])
def test_full_depth_first_minibatch(k):
    """All layers of the configuration (and the LM head of configuration 4):
    F0, B0, A0, U0 with every output compared in full."""
    w = W.CONFIGS[k]
    print(f"\n[cfg{k} full depth, first minibatch] start", flush=True)
    rep = run_parity(w, threshold=1, n_minibatches=1, verbose=True, cfg_kw=dict(act_slots=1, stash_slots=1))
    _show(f"cfg{k} full depth", rep)
    assert rep["ok"], worst_entries(rep)
    assert rep["events"] == 4


@pytest.mark.timeout(900)
def test_config2_whole_schedule_two_windows_stashed():
    w = W.CONFIGS[2]
    print("\n[cfg2 whole schedule, 2 windows, stashed] start", flush=True)
    rep = run_parity(w, n_windows=2, policy=OSched.STASHED, verbose=True)
    _show("cfg2 schedule stashed", rep)
    assert rep["ok"], worst_entries(rep)
    assert rep["max_resident_versions"] == 2          # an older version stays across each update


@pytest.mark.timeout(900)
def test_config2_schedule_current_weights_in_backward():
    """One window, its update, and the minibatches whose forward ran before it:
    their backward reads the version published in between."""
    w = W.CONFIGS[2]
    print("\n[cfg2 schedule, current weights in backward] start", flush=True)
    ev = OSched.generate(w.depth, w.pipelines, w.stage, w.threshold, w.threshold + w.act_slots, w.inject_limit,
                         OSched.NEXT_BUBBLE, OSched.CURRENT)
    fwd = {e.mb: e.version for e in ev if e.kind == OSched.F}
    assert sum(1 for e in ev if e.kind == OSched.B and e.version != fwd[e.mb]) >= 4
    rep = run_parity(w, n_minibatches=w.threshold + w.act_slots, policy=OSched.CURRENT, verbose=True)
    _show("cfg2 schedule current", rep)
    assert rep["ok"], worst_entries(rep)


@pytest.mark.timeout(900)
def test_config5_width_three_stashed_versions():
    """Configuration 5's width, sequence length and stash capacity (three older
    versions beside the current one) at one layer. The event list is written
    by hand -- the stage library takes its version tags from the list, whoever
    produced it: after three updates, minibatches 0, 2, 4 still await their
    backward with versions 0, 1, 2 while version 3 is current, then each
    backward selects its own version."""
    E = OSched.Event
    F, B, A, U = OSched.F, OSched.B, OSched.A, OSched.U
    ev = []
    for u in range(3):          # F(2u), F(2u+1) at version u; B(2u+1), A, U -> version u+1; mb 2u stays in flight
        ev += [E(F, 0, 0, 2 * u, u), E(F, 0, 0, 2 * u + 1, u), E(B, 0, 0, 2 * u + 1, u), E(A, 0, 0, 2 * u + 1, 0),
               E(U, 0, 0, u, u + 1)]
    ev += [E(F, 0, 0, 6, 3)]
    for mb, v in ((0, 0), (2, 1), (4, 2), (6, 3)):
        ev += [E(B, 0, 0, mb, v), E(A, 0, 0, mb, 0)]
    ev += [E(U, 0, 0, 3, 4)]
    w = W.CONFIGS[5].with_(n_layers=1, lr=1e-3)
    print("\n[cfg5 width, three stashed versions] start", flush=True)
    rep = run_parity(w, threshold=1, events=ev, verbose=True, cfg_kw=dict(act_slots=5, stash_slots=3))
    _show("cfg5 stash3", rep)
    assert rep["ok"], worst_entries(rep)
    assert rep["max_resident_versions"] == 4


@pytest.mark.timeout(900)
@pytest.mark.parametrize("key", ["paper_gpt_h1600", "paper_bert_h1600"])
def test_paper_shaped_one_layer(key):
    """Hidden size 1600 (Table 2): multiples of 64 that are not multiples of
    128, 25 heads of 64 (fused attention) or 32 heads of 50 (unfused attention
    on the generic kernels, heads not 16-byte aligned)."""
    w = W.PAPER[key].with_(n_layers=1)
    print(f"\n[{key} one layer at full width] start", flush=True)
    rep = run_parity(w, threshold=1, n_minibatches=1, verbose=True,
                     cfg_kw=dict(act_slots=1, stash_slots=1))
    _show(key, rep)
    assert rep["ok"], worst_entries(rep)


@pytest.mark.timeout(900)
def test_full_width_first_stage():
    """Configuration 2's width with the input embedding in front (GPT-2's
    50257-row vocabulary, 4096 token ids per minibatch): one layer, one
    minibatch through forward, backward, accumulate, update."""
    w = W.FIRST["first_gpt_d1024"].with_(n_layers=1)
    print("\n[first stage, one layer at full width] start", flush=True)
    rep = run_parity(w, threshold=1, n_minibatches=1, verbose=True, cfg_kw=dict(act_slots=1, stash_slots=1))
    _show("first stage", rep)
    assert rep["ok"], worst_entries(rep)


@pytest.mark.timeout(600)
def test_streaming_kernels_largest_config():
    """cfg5: 805,519,360 parameters. G after two accumulations and theta, m, v
    and the published bf16 version after the update, on sampled entries."""
    import torch
    w = W.CONFIGS[5]
    print("\n[cfg5 streaming kernels] start", flush=True)
    gpu = GpuStage(w, act_slots=2, stash_slots=1)
    n = gpu.n
    assert not gpu.stage.amdp_stage_get_overlap(), "d_model 4096: the side stream is off by default"
    import paper_2605_29664_amd as amdp
    layout = amdp.amdp_stage_param_layout(gpu.cfg)
    gen = torch.Generator(device="cuda").manual_seed(296645)
    theta = torch.randn(n, device="cuda", generator=gen, dtype=torch.float32) * 0.02
    m = torch.randn(n, device="cuda", generator=gen, dtype=torch.float32) * 1e-5
    v = torch.rand(n, device="cuda", generator=gen, dtype=torch.float32) * 1e-10
    gpu.stage.amdp_stage_set_state(theta, m, v, 9, 4)
    chk = torch.empty(n, dtype=torch.float32, device="cuda")
    gpu.stage.amdp_stage_get_state(chk, None, None, None)
    torch.cuda.synchronize()
    assert torch.equal(chk, theta), "master differs from what was loaded"
    del chk
    idx = torch.cat([torch.arange(0, 4096), torch.arange(n - 4096, n),
                     torch.randint(0, n, (200000,), generator=torch.Generator().manual_seed(5))]).cuda()
    gs = []
    g = torch.empty(n, dtype=torch.float32, device="cuda")
    for mb in range(2):
        X = gpu.to_dev(W.make_x(w, mb), gpu.dt)
        dY = gpu.to_dev(W.make_dy(w, mb), gpu.dt)
        Y = torch.empty_like(X)
        assert not bool(torch.isnan(X.float()).any())
        gpu.stage.amdp_stage_forward(mb, 4, X, None, Y)
        torch.cuda.synchronize()
        assert not bool(torch.isnan(Y.float()).any()), "forward produced NaN"
        gpu.stage.amdp_stage_backward(mb, 4, dY, None)
        gpu.stage.amdp_stage_get_staged_grad(g)
        torch.cuda.synchronize()
        bad = [(name, int(torch.isnan(g[off:off + r * c]).sum())) for name, off, r, c in layout
               if bool(torch.isnan(g[off:off + r * c]).any())]
        assert not bad, (mb, int(torch.isnan(Y.float()).sum()), bad)
        gs.append(g[idx].double().cpu().numpy())
        gpu.stage.amdp_grad_accumulate(mb)
    G = torch.empty(n, dtype=torch.float32, device="cuda")
    gpu.stage.amdp_stage_get_state(None, None, None, G)
    torch.cuda.synchronize()
    G_s = G[idx].double().cpu().numpy()
    assert np.array_equal(G_s, (gs[0].astype(np.float32) + gs[1].astype(np.float32)).astype(np.float64))
    th_s, m_s, v_s = (t[idx].double().cpu().numpy() for t in (theta, m, v))
    nv = gpu.update(w, 0.5)
    th2, m2, v2 = (torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(3))
    step, ver = gpu.stage.amdp_stage_get_state(th2, m2, v2, G)
    torch.cuda.synchronize()
    assert (nv, step, ver) == (5, 10, 5)
    ref_th, ref_m, ref_v = optim.adam_step(th_s, m_s, v_s, G_s, 10, w.lr, w.beta1, w.beta2, w.eps, grad_scale=0.5)
    assert rel_err(th2[idx].cpu().numpy(), ref_th) <= 1e-6
    assert rel_err(m2[idx].cpu().numpy(), ref_m) <= 1e-6
    assert rel_err(v2[idx].cpu().numpy(), ref_v) <= 1e-6
    assert rel_err((th2[idx].double().cpu().numpy() - th_s), ref_th - th_s) <= 1e-3
    assert float(G.abs().max()) == 0.0
    # the published version is the bf16 rounding of the new master: a forward
    # with it must equal a forward after reloading that master as a fresh state
    X = gpu.to_dev(W.make_x(w, 7), gpu.dt)
    Y1, Y2 = torch.empty_like(X), torch.empty_like(X)
    gpu.stage.amdp_stage_forward(100, 5, X, None, Y1)
    gpu.stage.amdp_stage_set_state(th2, m2, v2, 10, 5)
    gpu.stage.amdp_stage_forward(101, 5, X, None, Y2)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)
    gpu.stage.close()


def _run_schedule_on_device(w, policy, fused, M, lr):
    """Runs M minibatches of w's schedule with device-resident inputs (a ring of four) and
    returns every backward's dX plus the final state, all as device tensors."""
    import torch
    import paper_2605_29664_amd as amdp
    gpu = GpuStage(w, act_slots=w.act_slots, stash_slots=max(2, w.stash_slots))
    layout = amdp.amdp_stage_param_layout(gpu.cfg)
    gpu.set_state(W.make_theta(w, layout))
    gpu.stage.amdp_stage_set_fused_accumulate(fused)
    ring = 4
    X = [gpu.to_dev(W.make_x(w, k), gpu.dt) for k in range(ring)]
    dY = [None if w.has_lm_head else gpu.to_dev(W.make_dy(w, k), gpu.dt) for k in range(ring)]
    aux = [None if W.make_aux(w, k) is None else gpu.to_dev(np.asarray(W.make_aux(w, k), dtype=np.int32)) for k in range(ring)]
    out = torch.empty(1, dtype=torch.float32, device="cuda:0") if w.has_lm_head else torch.empty_like(X[0])
    ev = amdp.amdp_schedule_generate(w.depth, w.pipelines, w.stage, w.threshold, M, w.inject_limit, amdp.U_NEXT_BUBBLE, policy)
    dxs = {}
    for e in ev:
        r = e.mb % ring
        if e.kind == amdp.EV_F:
            gpu.stage.amdp_stage_forward(e.mb, e.version, X[r], aux[r], out)
        elif e.kind == amdp.EV_B:
            dx = torch.empty_like(X[0])
            gpu.stage.amdp_stage_backward(e.mb, e.version, dY[r], dx)
            dxs[e.mb] = dx
        elif e.kind == amdp.EV_A:
            gpu.stage.amdp_grad_accumulate(e.mb)
        else:
            gpu.stage.amdp_apply_update(lr, w.beta1, w.beta2, w.eps, w.weight_decay, 1.0 / w.threshold, True)
    n = gpu.n
    st = [torch.empty(n, dtype=torch.float32, device="cuda:0") for _ in range(4)]
    gpu.stage.amdp_stage_get_state(*st)
    torch.cuda.synchronize()
    gpu.stage.close()
    return ev, dxs, st


@pytest.mark.timeout(600)
@pytest.mark.parametrize("k", [3, 4, 5])
def test_full_size_schedule_properties(k):
    """Configurations 3, 4, 5 at full depth through one window, its update and the
    minibatches in flight across it, checked by properties that need no oracle:
    (a) with the accumulation fused into backward the final state is bit-identical;
    (b) with the current version in backward instead of the forward's, exactly the
        minibatches whose forward ran before the update and whose backward ran after
        it get a different dX (Section 3.1's mismatched minibatches), every other dX is
        bit-identical, and the state after the update differs."""
    import torch
    from oracle import schedule as OS
    w = W.CONFIGS[k]
    M = w.threshold + w.act_slots + 2
    print(f"\n[cfg{k} schedule properties, {M} minibatches] start", flush=True)
    ev_s, dx_s, st_s = _run_schedule_on_device(w, OS.STASHED, False, M, 1e-3)
    print("  stashed done", flush=True)
    ev_f, dx_f, st_f = _run_schedule_on_device(w, OS.STASHED, True, M, 1e-3)
    print("  fused done", flush=True)
    for a, b in zip(st_s, st_f):
        assert torch.equal(a, b), "fused accumulation changed the state"
    for mb in dx_s:
        assert torch.equal(dx_s[mb], dx_f[mb])
    del dx_f, st_f
    ev_c, dx_c, st_c = _run_schedule_on_device(w, OS.CURRENT, False, M, 1e-3)
    print("  current done", flush=True)
    fwd = {e.mb: e.version for e in ev_c if e.kind == OS.F}
    mismatched = {e.mb for e in ev_c if e.kind == OS.B and e.version != fwd[e.mb]}
    assert len(mismatched) >= 1 and len(mismatched) <= w.act_slots
    # The first update closes window 0, none of whose minibatches is mismatched, so version 1 is
    # the same in both runs: every backward whose two versions agree must give the same dX bit for
    # bit, before and after that update, and every mismatched one a different dX.
    for e in ev_c:
        if e.kind != OS.B:
            continue
        same = torch.equal(dx_s[e.mb], dx_c[e.mb])
        if e.mb in mismatched:
            assert not same, f"minibatch {e.mb}: backward with a newer version gave the same dX"
        else:
            assert same, f"minibatch {e.mb}: dX differs although its versions agree"
    assert all(torch.isfinite(t).all() for t in st_c)
    assert not torch.equal(st_s[0], st_c[0])       # the last update applied different gradients
