"""GPU parity at the benchmark's full widths. The fp64 oracle needs minutes
for a whole stage, so these tests compare (a) ONE layer at the full width,
sequence length and microbatch of each configuration -- the same GEMM,
attention and row-kernel launch shapes bench.py times -- through a complete
forward / backward / accumulate / update, and (b) the full-depth forward on
outputs the oracle can compute by themselves: one whole sequence (attention
never mixes sequences) or a causal prefix of it (a causal block's output at
position p depends on positions <= p only); (c) the streaming kernels on the
largest configuration's 805 M parameters, on sampled entries."""
import numpy as np
import pytest

import workloads as W
from oracle import optim
from oracle.stage import Stage as OStage
from tests.parity import run_parity, worst_entries, GpuStage, rel_err, TOL

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(900)
@pytest.mark.parametrize("k", [2, 3, 5, 4])
def test_full_width_one_layer(k):
    w = W.CONFIGS[k].with_(n_layers=1)
    print(f"\n[cfg{k} one layer at full width] start", flush=True)
    rep = run_parity(w, threshold=1, n_minibatches=1, verbose=True,
                     cfg_kw=dict(act_slots=1, stash_slots=1))
    print(f"[cfg{k} one layer] worst={rep['worst']:.3e} {rep['seconds']:.0f}s", worst_entries(rep, 4), flush=True)
    assert rep["ok"], worst_entries(rep)


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
    print(f"[{key} one layer] worst={rep['worst']:.3e} {rep['seconds']:.0f}s", worst_entries(rep, 4), flush=True)
    assert rep["ok"], worst_entries(rep)


@pytest.mark.timeout(900)
def test_full_width_first_stage():
    """Configuration 2's width with the input embedding in front (GPT-2's
    50257-row vocabulary, 4096 token ids per minibatch): one layer, one
    minibatch through forward, backward, accumulate, update."""
    w = W.FIRST["first_gpt_d1024"].with_(n_layers=1)
    print("\n[first stage, one layer at full width] start", flush=True)
    rep = run_parity(w, threshold=1, n_minibatches=1, verbose=True, cfg_kw=dict(act_slots=1, stash_slots=1))
    print(f"[first stage] worst={rep['worst']:.3e} {rep['seconds']:.0f}s", worst_entries(rep, 4), flush=True)
    assert rep["ok"], worst_entries(rep)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("k,prefix", [(2, 1024), (3, 512), (5, 256)])
def test_full_depth_forward_one_sequence(k, prefix):
    w = W.CONFIGS[k]
    print(f"\n[cfg{k} full depth forward, sequence 0, first {prefix} positions] start", flush=True)
    full = OStage.from_workload(w)
    theta0 = W.make_theta(w, full.layout)
    x = W.make_x(w, 0)
    aux = W.make_valid_len(w, 0) if w.block_kind == 1 else None
    gpu = GpuStage(w, act_slots=1, stash_slots=1)
    gpu.set_state(theta0)
    y = gpu.forward(0, 0, x, aux)
    gpu.stage.close()
    # oracle: sequence 0 alone, truncated to `prefix` positions (exact for the rows compared)
    sub = OStage(w.block_kind, w.n_layers, w.d_model, w.n_heads, w.d_ffn, prefix, 1, ln_eps=w.ln_eps)
    version = optim.round_to_bf16(theta0)
    sub_aux = None if aux is None else np.minimum(aux[:1], prefix)
    if aux is not None:
        assert prefix == w.seq_len          # padding masks need the whole sequence
    y_ref, _ = sub.forward(version, x[:prefix], sub_aux)
    err = rel_err(y[:prefix], y_ref)
    print(f"[cfg{k} full depth forward] rel err {err:.3e}", flush=True)
    assert err <= TOL[w.dtype]


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
