"""Parity harness: drives the HIP library (through its C ABI binding) and the
CPU oracle with identical seeded inputs over one schedule, and compares every
result event by event. Used by the GPU tests and by __graft_entry__.smoke().

Two gates per compared tensor (Y, dX, every parameter's slice of g, G, m, v,
theta, the loss):
  * norm-wise   ||x - ref||_F / ||ref||_F        <= TOL[dtype]
  * element-wise max|x - ref| / rms(ref != 0)    <= ELEM_TOL[dtype]
The second one is there so that a few wrong rows or a wrong last tile cannot
hide inside the norm of a large tensor: one entry that is off by the tensor's
own typical magnitude fails it.

At every update the library's Adam step is also checked against the oracle's
step applied to the LIBRARY's own state before the update (same G, m, v, theta
in, so no bf16 noise enters): the change of theta must agree to 1e-3, m and v
to 1e-6, and the published 16-bit version must be the round-to-nearest-even of
the new master bit for bit. (theta against the free-running oracle is compared
norm-wise over the whole vector only; see the comment at the update.)"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402
from oracle import optim as OOptim  # noqa: E402
from oracle import schedule as OSched  # noqa: E402
from oracle.run import StageRun  # noqa: E402
from oracle.stage import Stage as OracleStage  # noqa: E402

# norm-wise relative tolerances: ||x - ref||_F / ||ref||_F per compared tensor
TOL = {W.configs.BF16: 2e-2, W.configs.FP32: 1e-5}
# element-wise: max |x - ref| <= ELEM_TOL * rms(ref). bf16: an output of typical size rms is
# rounded to 8 bits (relative 2^-9 = 2e-3 each, the largest entries of a normal-like tensor are
# ~5 rms, so rounding alone reaches 1e-2 rms) and its inputs carry the same rounding through
# products of hundreds to thousands of terms; measured maxima over all test shapes and the five
# configurations at full depth: 0.19 (bf16), 1.9e-5 (fp32). An entry replaced by an unrelated
# one is off by ~1.4 rms on average, and the largest of a wrong row's entries by 3 rms or more.
# rms is taken over the entries of ref that are not exactly zero, so that a tensor that is zero
# by structure almost everywhere (the token embedding's gradient) is measured in units of its
# populated entries.
ELEM_TOL = {W.configs.BF16: 0.5, W.configs.FP32: 2e-4}
# Adam step with identical inputs on both sides (fp32 kernel against the fp64 oracle)
UPDATE_SAME_INPUT_TOL = dict(delta_theta=1e-3, moments=1e-6)


def rel_err(x, ref):
    x = np.asarray(x, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    den = np.linalg.norm(ref)
    num = np.linalg.norm(x - ref)
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return float(num / den)


def elem_err(x, ref):
    """max |x - ref| in units of the rms of ref's non-zero entries."""
    x = np.asarray(x, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.sum(ref * ref) / max(1, np.count_nonzero(ref))))
    num = float(np.max(np.abs(x - ref)))
    if not np.isfinite(num):
        return float("inf")
    if rms == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / rms


def make_cfg(w, **kw):
    from paper_2605_29664_amd import binding
    return binding.make_config(**W.stage_config_args(w, **kw))


aux_for = W.make_aux


class GpuStage:
    """The library side of a parity run: host arrays in, host arrays out."""

    def __init__(self, w, device="cuda:0", poison=False, options=None, **cfg_kw):
        import torch
        import paper_2605_29664_amd as amdp
        self.torch, self.amdp, self.w = torch, amdp, w
        self.dev = torch.device(device)
        self.cfg = make_cfg(w, **cfg_kw)
        self.stage = amdp.Stage(self.cfg, device=device, poison=poison)
        for opt, val in (options or {}).items():
            self.stage.amdp_stage_set_option(opt, val)
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
        X = None if x is None else self.to_dev(x, self.dt)
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

    def state(self, which=("theta", "m", "v", "G")):
        torch = self.torch
        bufs = {k: torch.empty(self.n, dtype=torch.float32, device=self.dev) for k in which}
        step, ver = self.stage.amdp_stage_get_state(*(bufs.get(k) for k in ("theta", "m", "v", "G")))
        torch.cuda.synchronize()
        out = {k: b.cpu().numpy() for k, b in bufs.items()}
        out.update(step=step, version=ver)
        return out

    def read_version(self, version):
        """The published weights of a resident version, as float32 values."""
        torch = self.torch
        buf = torch.empty(self.n + 1, dtype=self.dt, device=self.dev)
        self.stage.amdp_stage_read_version(version, buf)
        torch.cuda.synchronize()
        return buf[:self.n].float().cpu().numpy()


def run_parity(w, n_windows=2, policy=OSched.STASHED, placement=OSched.NEXT_BUBBLE, inject_limit=None,
               threshold=None, n_minibatches=None, verbose=True, tol=None, cfg_kw=None, device="cuda:0",
               aux_fn=None, options=None, events=None, elem_tol=None):
    """Runs M = n_windows*T + w*P minibatches through library and oracle (or the
    hand-written `events`, a list of oracle-schedule Event records).
    Returns {'ok', 'worst', 'worst_elem', 'details': [(event, name, err, elem)], ...}."""
    import paper_2605_29664_amd as amdp
    tol = tol if tol is not None else TOL[w.dtype]
    etol = elem_tol if elem_tol is not None else ELEM_TOL[w.dtype]
    T = threshold or w.threshold
    n_inj = inject_limit or w.inject_limit
    M = n_minibatches if n_minibatches is not None else n_windows * T + min(n_inj, w.depth - w.stage) * w.pipelines
    ost = OracleStage.from_workload(w)
    theta0 = W.make_theta(w, ost.layout)
    storage = "bf16" if w.dtype == W.configs.BF16 else "fp32"
    orun = StageRun(ost, theta0, storage=storage, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                    weight_decay=w.weight_decay, grad_scale=1.0 / T)

    if events is None:
        ev_lib = amdp.amdp_schedule_generate(w.depth, w.pipelines, w.stage, T, M, n_inj, placement, policy)
        ev_ref = OSched.generate(w.depth, w.pipelines, w.stage, T, M, n_inj, placement, policy)
        sched_equal = [(e.kind, e.pipeline, e.flags, e.mb, e.version) for e in ev_lib] == [tuple(e) for e in ev_ref]
    else:
        ev_lib = ev_ref = list(events)
        sched_equal = True

    kw = dict(cfg_kw or {})
    stats = OSched.stats(ev_ref, T)
    kw.setdefault("act_slots", max(1, stats["max_inflight"]))
    kw.setdefault("stash_slots", max(w.stash_slots, stats["max_live_versions"] - 1, 1))
    gpu = GpuStage(w, device=device, options=options, **kw)
    gpu.set_state(theta0)

    details = []
    worst = 0.0
    worst_elem = 0.0
    max_resident = 1
    t0 = time.time()

    def note(ev, name, x, ref, gate_tol=None):
        """Records both error measures of one tensor; gate_tol = (norm-wise, element-wise)
        overrides the run's tolerances for this entry (errors are stored relative to the
        run's tolerances so that one pair of maxima decides)."""
        nonlocal worst, worst_elem
        e, m = rel_err(x, ref), elem_err(x, ref)
        if gate_tol is not None:
            e = e * (tol / gate_tol[0])
            m = m * (etol / gate_tol[1]) if gate_tol[1] else 0.0
        details.append((f"{OSched.KIND_NAMES[ev.kind]}{ev.mb}", name, e, m))
        worst = max(worst, e) if np.isfinite(e) else float("inf")
        worst_elem = max(worst_elem, m) if np.isfinite(m) else float("inf")

    def note_slices(ev, prefix, x, ref, **kwargs):
        for name, off, r, c in ost.layout:
            note(ev, prefix + name, x[off:off + r * c], ref[off:off + r * c], **kwargs)

    resident_ok = True
    for ev in ev_lib:
        if verbose:
            print(f"  {OSched.KIND_NAMES[ev.kind]}{ev.mb} ...", flush=True)
        if ev.kind == amdp.EV_F:
            x = None if w.has_embedding else W.make_x(w, ev.mb)
            aux = (aux_fn or aux_for)(w, ev.mb)
            ref = orun.forward(ev.mb, ev.version, x, aux)
            got = gpu.forward(ev.mb, ev.version, x, aux)
            note(ev, "loss" if w.has_lm_head else "Y", got, ref)
        elif ev.kind == amdp.EV_B:
            dy = None if w.has_lm_head else W.make_dy(w, ev.mb)
            dx_ref, g_ref = orun.backward(ev.mb, ev.version, dy)
            dx, g = gpu.backward(ev.mb, ev.version, dy)
            if not w.has_embedding:
                note(ev, "dX", dx, dx_ref)
            note_slices(ev, "g.", g, g_ref)
        elif ev.kind == amdp.EV_A:
            orun.accumulate(ev.mb)
            gpu.accumulate(ev.mb)
            note_slices(ev, "G.", gpu.state(("G",))["G"], orun.G)
        else:
            s0 = gpu.state()
            orun.update()
            nv = gpu.update(w, 1.0 / T)
            s = gpu.state()
            note_slices(ev, "m.", s["m"], orun.m)
            # v is the square of the gradient: its largest entries are many rms of v, and an
            # error of the gradient is multiplied by them; norm-wise only (element-wise the
            # gradient sum itself is gated at every accumulation, v's arithmetic just below)
            note_slices(ev, "v.", s["v"], orun.v, gate_tol=(tol, None))
            # theta against the free-running oracle over the whole vector, norm-wise only: Adam
            # divides by |g|, so where a gradient is zero up to rounding noise (the key bias:
            # softmax ignores a constant added to a row of scores) both sides step by lr times a
            # random sign, which is noise of size lr in that slice and says nothing about the
            # kernel. What pins the update itself is the same-input comparison below.
            note(ev, "theta", s["theta"], orun.theta, gate_tol=(tol, None))
            # the kernel's step against the oracle's step from the library's own state
            th, m_, v_ = OOptim.adam_step(s0["theta"].astype(np.float64), s0["m"].astype(np.float64),
                                          s0["v"].astype(np.float64), s0["G"].astype(np.float64), s0["step"] + 1,
                                          w.lr, w.beta1, w.beta2, w.eps, weight_decay=w.weight_decay,
                                          grad_scale=1.0 / T)
            d0 = s0["theta"].astype(np.float64)
            upd = UPDATE_SAME_INPUT_TOL
            note(ev, "delta_theta|same inputs", s["theta"] - d0, th - d0, gate_tol=(upd["delta_theta"], None))
            note(ev, "m|same inputs", s["m"], m_, gate_tol=(upd["moments"], None))
            note(ev, "v|same inputs", s["v"], v_, gate_tol=(upd["moments"], None))
            if np.any(s0["G"] != 0.0) and not np.any(s["theta"] != s0["theta"]):
                note(ev, "update changed nothing", np.ones(1), np.zeros(1))
            pub = gpu.read_version(nv)
            want = OOptim.round_to_bf16(s["theta"]) if storage == "bf16" else s["theta"]
            if not np.array_equal(pub, want.astype(np.float32)):
                note(ev, "published version != round(master)", np.ones(1), np.zeros(1))
            if nv != orun.version or s["step"] != orun.step or np.any(s["G"] != 0.0):
                resident_ok = False
        res = gpu.stage.amdp_stage_resident_versions()
        max_resident = max(max_resident, len(res))
        if res != sorted(orun.versions):
            resident_ok = False
        if verbose and ev.kind in (amdp.EV_B, amdp.EV_U):
            print(f"  {details[-1][0]}: worst so far {worst:.3e} (element-wise {worst_elem:.3e})", flush=True)
    rep = dict(ok=bool(sched_equal and resident_ok and worst <= tol and worst_elem <= etol), worst=worst,
               worst_elem=worst_elem, tol=tol, elem_tol=etol,
               schedule_equal=sched_equal, residency_equal=resident_ok, events=len(ev_lib),
               max_resident_versions=max_resident, seconds=time.time() - t0, details=details)
    gpu.stage.close()
    return rep


def worst_entries(rep, k=8):
    by_norm = sorted(rep["details"], key=lambda d: -d[2] if np.isfinite(d[2]) else -1e300)[:k]
    by_elem = sorted(rep["details"], key=lambda d: -d[3] if np.isfinite(d[3]) else -1e300)[:max(2, k // 2)]
    return {"norm": by_norm, "elem": by_elem}
