"""Parity harness: drives the HIP library (through its C ABI binding) and the
CPU oracle with identical seeded inputs over one schedule, and compares every
result event by event. Used by the GPU tests and by __graft_entry__.smoke()."""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402
from oracle import schedule as OSched  # noqa: E402
from oracle.run import StageRun  # noqa: E402
from oracle.stage import Stage as OracleStage  # noqa: E402

# norm-wise relative tolerances: ||x - ref||_F / ||ref||_F per compared tensor
TOL = {W.configs.BF16: 2e-2, W.configs.FP32: 1e-5}


def rel_err(x, ref):
    x = np.asarray(x, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    den = np.linalg.norm(ref)
    num = np.linalg.norm(x - ref)
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return float(num / den)


def make_cfg(w, **kw):
    from paper_2605_29664_amd import binding
    args = dict(block_kind=w.block_kind, n_layers=w.n_layers, d_model=w.d_model, n_heads=w.n_heads,
                d_ffn=w.d_ffn, seq_len=w.seq_len, microbatch=w.microbatch, dtype=w.dtype,
                has_lm_head=w.has_lm_head, vocab=w.vocab, ln_eps=w.ln_eps, act_slots=w.act_slots,
                stash_slots=w.stash_slots, has_embedding=w.has_embedding)
    args.update(kw)
    return binding.make_config(**args)


def aux_for(w, mb):
    if w.has_lm_head:
        return W.make_targets(w, mb)
    if w.has_embedding:          # token ids, then the padding mask for the bidirectional block
        t = W.make_tokens(w, mb)
        return np.concatenate([t, W.make_valid_len(w, mb)]) if w.block_kind == W.configs.BERT_POSTLN_BIDIR else t
    if w.block_kind == W.configs.BERT_POSTLN_BIDIR:
        return W.make_valid_len(w, mb)
    return None


class GpuStage:
    """The library side of a parity run: host arrays in, host arrays out."""

    def __init__(self, w, device="cuda:0", poison=False, **cfg_kw):
        import torch
        import paper_2605_29664_amd as amdp
        self.torch, self.amdp, self.w = torch, amdp, w
        self.dev = torch.device(device)
        self.cfg = make_cfg(w, **cfg_kw)
        self.stage = amdp.Stage(self.cfg, device=device, poison=poison)
        self.n = self.stage.n_params
        self.dt = self.stage.act_dtype
        self.keep = {}     # device tensors that must outlive the enqueued work

    def to_dev(self, a, dtype=None):
        t = self.torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)
        return t.to(dtype) if dtype is not None else t

    def set_state(self, theta, m=None, v=None, step=0, version=0):
        f32 = self.torch.float32
        self.stage.amdp_stage_set_state(self.to_dev(theta, f32), None if m is None else self.to_dev(m, f32),
                                        None if v is None else self.to_dev(v, f32), step, version)
        self.torch.cuda.synchronize()

    def forward(self, mb, version, x, aux):
        torch = self.torch
        X = self.to_dev(x, self.dt)
        A = None if aux is None else self.to_dev(np.asarray(aux, dtype=np.int32))
        if self.w.has_lm_head:
            out = torch.empty(1, dtype=torch.float32, device=self.dev)
        else:
            out = torch.empty((self.w.tokens, self.w.d_model), dtype=self.dt, device=self.dev)
        self.stage.amdp_stage_forward(mb, version, X, A, out)
        torch.cuda.synchronize()
        r = out.float().cpu().numpy()
        return float(r[0]) if self.w.has_lm_head else r

    def backward(self, mb, version, dy):
        torch = self.torch
        dY = None if dy is None else self.to_dev(dy, self.dt)
        dX = torch.empty((self.w.tokens, self.w.d_model), dtype=self.dt, device=self.dev)
        self.stage.amdp_stage_backward(mb, version, dY, dX)
        g = torch.empty(self.n, dtype=torch.float32, device=self.dev)
        self.stage.amdp_stage_get_staged_grad(g)
        torch.cuda.synchronize()
        return dX.float().cpu().numpy(), g.cpu().numpy()

    def accumulate(self, mb):
        self.stage.amdp_grad_accumulate(mb)

    def update(self, w, grad_scale):
        return self.stage.amdp_apply_update(w.lr, w.beta1, w.beta2, w.eps, w.weight_decay, grad_scale, True)

    def state(self):
        torch = self.torch
        bufs = [torch.empty(self.n, dtype=torch.float32, device=self.dev) for _ in range(4)]
        step, ver = self.stage.amdp_stage_get_state(*bufs)
        torch.cuda.synchronize()
        th, m, v, G = (b.cpu().numpy() for b in bufs)
        return dict(theta=th, m=m, v=v, G=G, step=step, version=ver)


def run_parity(w, n_windows=2, policy=OSched.STASHED, placement=OSched.NEXT_BUBBLE, inject_limit=None,
               threshold=None, n_minibatches=None, verbose=True, tol=None, cfg_kw=None, device="cuda:0",
               aux_fn=None):
    """Runs M = n_windows*T + w*P minibatches through library and oracle.
    Returns {'ok', 'worst', 'details': [(event, name, err)], ...}."""
    import paper_2605_29664_amd as amdp
    tol = tol if tol is not None else TOL[w.dtype]
    T = threshold or w.threshold
    n_inj = inject_limit or w.inject_limit
    M = n_minibatches if n_minibatches is not None else n_windows * T + min(n_inj, w.depth - w.stage) * w.pipelines
    ost = OracleStage.from_workload(w)
    theta0 = W.make_theta(w, ost.layout)
    storage = "bf16" if w.dtype == W.configs.BF16 else "fp32"
    orun = StageRun(ost, theta0, storage=storage, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                    weight_decay=w.weight_decay, grad_scale=1.0 / T)

    ev_lib = amdp.amdp_schedule_generate(w.depth, w.pipelines, w.stage, T, M, n_inj, placement, policy)
    ev_ref = OSched.generate(w.depth, w.pipelines, w.stage, T, M, n_inj, placement, policy)
    sched_equal = [(e.kind, e.pipeline, e.flags, e.mb, e.version) for e in ev_lib] == [tuple(e) for e in ev_ref]

    kw = dict(cfg_kw or {})
    stats = OSched.stats(ev_ref, T)
    kw.setdefault("act_slots", max(1, stats["max_inflight"]))
    kw.setdefault("stash_slots", max(w.stash_slots, stats["max_live_versions"] - 1, 1))
    gpu = GpuStage(w, device=device, **kw)
    gpu.set_state(theta0)

    details = []
    worst = 0.0
    t0 = time.time()

    def note(ev, name, err):
        nonlocal worst
        details.append((f"{OSched.KIND_NAMES[ev.kind]}{ev.mb}", name, err))
        if not np.isfinite(err) or err > worst:
            worst = err if np.isfinite(err) else float("inf")

    resident_ok = True
    for ev in ev_lib:
        if verbose:
            print(f"  {OSched.KIND_NAMES[ev.kind]}{ev.mb} ...", flush=True)
        if ev.kind == amdp.EV_F:
            x, aux = W.make_x(w, ev.mb), (aux_fn or aux_for)(w, ev.mb)
            ref = orun.forward(ev.mb, ev.version, x, aux)
            got = gpu.forward(ev.mb, ev.version, x, aux)
            note(ev, "loss" if w.has_lm_head else "Y", rel_err(got, ref))
        elif ev.kind == amdp.EV_B:
            dy = None if w.has_lm_head else W.make_dy(w, ev.mb)
            dx_ref, g_ref = orun.backward(ev.mb, ev.version, dy)
            dx, g = gpu.backward(ev.mb, ev.version, dy)
            note(ev, "dX", rel_err(dx, dx_ref))
            for name, off, r, c in ost.layout:
                note(ev, "g." + name, rel_err(g[off:off + r * c], g_ref[off:off + r * c]))
        elif ev.kind == amdp.EV_A:
            orun.accumulate(ev.mb)
            gpu.accumulate(ev.mb)
            note(ev, "G", rel_err(gpu.state()["G"], orun.G))
        else:
            theta_before = orun.theta.copy()
            orun.update()
            nv = gpu.update(w, 1.0 / T)
            s = gpu.state()
            note(ev, "m", rel_err(s["m"], orun.m))
            note(ev, "v", rel_err(s["v"], orun.v))
            note(ev, "theta", rel_err(s["theta"], orun.theta))
            details.append((f"U{ev.mb}", "delta_theta(not gated)",
                            rel_err(s["theta"] - theta_before, orun.theta - theta_before)))
            if nv != orun.version or s["step"] != orun.step or np.any(s["G"] != 0.0):
                resident_ok = False
        if gpu.stage.amdp_stage_resident_versions() != sorted(orun.versions):
            resident_ok = False
        if verbose and ev.kind in (amdp.EV_B, amdp.EV_U):
            print(f"  {details[-1][0]}: worst so far {worst:.3e}", flush=True)
    rep = dict(ok=bool(sched_equal and resident_ok and worst <= tol), worst=worst, tol=tol,
               schedule_equal=sched_equal, residency_equal=resident_ok, events=len(ev_lib),
               seconds=time.time() - t0, details=details)
    gpu.stage.close()
    return rep


def worst_entries(rep, k=8):
    gated = [d for d in rep["details"] if "not gated" not in d[1]]
    return sorted(gated, key=lambda d: -d[2] if np.isfinite(d[2]) else -1e300)[:k]
