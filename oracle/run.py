"""Oracle: walk a stage's event list (forward / backward / accumulate / update)
and keep the state the method defines: the master parameters and Adam moments,
the running gradient sum of the open window, the weight versions that
in-flight minibatches still refer to, and each in-flight minibatch's saved
activations (Sections 3.1-3.3).

TEST INFRASTRUCTURE ONLY (see the package docstring).
"""
import numpy as np

from . import schedule as S
from . import optim
from .stage import Stage


class StageRun:
    def __init__(self, stage: Stage, theta0, storage="bf16", lr=1e-4, beta1=0.9, beta2=0.999,
                 eps=1e-8, weight_decay=0.0, grad_scale=1.0, bias_correction=True):
        """`storage` is the number type a weight version is published in:
        'bf16' (rounded copy of the fp32 master) or 'fp32'."""
        self.stage = stage
        self.theta = np.asarray(theta0, dtype=np.float64).copy()
        self.m = np.zeros_like(self.theta)
        self.v = np.zeros_like(self.theta)
        self.G = np.zeros_like(self.theta)
        self.step = 0
        self.version = 0
        self.hp = dict(lr=lr, beta1=beta1, beta2=beta2, eps=eps, weight_decay=weight_decay,
                       grad_scale=grad_scale, bias_correction=bias_correction)
        self._publish = optim.round_to_bf16 if storage == "bf16" else optim.round_to_fp32
        self.versions = {0: self._publish(self.theta)}
        self._pins = {}      # version -> in-flight minibatches whose forward read it
        self._fwd_version = {}
        self.saved = {}      # mb -> saved activations
        self.grads = {}      # mb -> per-minibatch flat gradient, until accumulated

    def forward(self, mb, version, x, aux=None):
        if mb in self.saved:
            raise RuntimeError("minibatch already in flight")
        out, saved = self.stage.forward(self.versions[version], x, aux)
        self.saved[mb] = saved
        self._fwd_version[mb] = version
        self._pins[version] = self._pins.get(version, 0) + 1
        return out

    def backward(self, mb, version, dy=None):
        dx, g = self.stage.backward(self.versions[version], self.saved[mb], dy)
        self.grads[mb] = g
        self._pins[self._fwd_version.pop(mb)] -= 1
        self._drop_unpinned()
        return dx, g

    def accumulate(self, mb):
        optim.accumulate(self.G, self.grads.pop(mb))
        del self.saved[mb]

    def update(self):
        self.step += 1
        self.theta, self.m, self.v = optim.adam_step(self.theta, self.m, self.v, self.G,
                                                     self.step, **self.hp)
        self.G = np.zeros_like(self.G)
        self.version += 1
        self.versions[self.version] = self._publish(self.theta)
        self._drop_unpinned()
        return self.version

    def _drop_unpinned(self):
        """The stash rule (Section 1 describes parameter stashing as keeping
        the forward's parameters for the matching backward): a version stays
        resident while it is current or while a minibatch whose forward read
        it still awaits its backward."""
        for v in list(self.versions):
            if v != self.version and self._pins.get(v, 0) == 0:
                del self.versions[v]

    def run(self, events, x_of, dy_of, aux_of=lambda mb: None, observer=None):
        """Execute an event list. x_of/dy_of/aux_of map a minibatch id to its
        inputs. `observer(event, payload)` sees every result."""
        for ev in events:
            if ev.kind == S.F:
                out = self.forward(ev.mb, ev.version, x_of(ev.mb), aux_of(ev.mb))
                payload = {"out": out}
            elif ev.kind == S.B:
                dx, g = self.backward(ev.mb, ev.version, dy_of(ev.mb))
                payload = {"dx": dx, "g": g}
            elif ev.kind == S.A:
                self.accumulate(ev.mb)
                payload = {"G": self.G}
            else:
                g_before = self.G.copy()
                self.update()
                payload = {"G_applied": g_before, "theta": self.theta, "m": self.m, "v": self.v,
                           "version": self.version}
            if observer is not None:
                observer(ev, payload)
