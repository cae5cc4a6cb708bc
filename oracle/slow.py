"""Loader for the oracle's scalar-loop tier (slow_stage.c): the same middle-stage
forward and backward as stage.py, written a second time as plain C loops over
scalars in double precision.

TEST INFRASTRUCTURE ONLY, like the rest of this package. It serves two ends:
the numpy tier is checked against an implementation that shares none of its
code (the tests compare the two to rounding-order differences), and the
benchmark reports it as the slowest CPU baseline. Middle stages only: no
embedding, no LM head.

The shared object is compiled with gcc on first use (and by the repository's
build step); it links nothing but libm.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slow_stage.c")
_SO = os.path.join(_HERE, "_slow_stage.so")
_lib = None


def build(force=False):
    """gcc -O2, no fast-math: the loops keep the order they are written in."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-std=c99", "-D_GNU_SOURCE", "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"], check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i, d, p = ctypes.c_int, ctypes.c_double, ctypes.c_void_p
        L.slow_saved_doubles_per_layer.restype = ctypes.c_long
        L.slow_saved_doubles_per_layer.argtypes = [i] * 5
        L.slow_stage_forward.restype = i
        L.slow_stage_forward.argtypes = [i] * 7 + [d] + [p] * 5
        L.slow_stage_backward.restype = i
        L.slow_stage_backward.argtypes = [i] * 7 + [d] + [p] * 5
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


class SlowStage:
    """Same shape record as stage.Stage (middle stages), same flat parameter order."""

    def __init__(self, block_kind, n_layers, d_model, n_heads, d_ffn, seq_len, microbatch, ln_eps=1e-5):
        self.shape = (int(block_kind), int(n_layers), int(d_model), int(n_heads), int(d_ffn), int(seq_len), int(microbatch))
        self.eps = float(ln_eps)
        _, L, D, H, F, s, b = self.shape
        self.N, self.D = s * b, D
        self.n_params = L * (12 * D * D + 13 * D) if F == 4 * D else L * (4 * D * D + 2 * D * F + 9 * D + F)
        self.saved_doubles = L * lib().slow_saved_doubles_per_layer(D, H, F, s, b)

    @classmethod
    def from_workload(cls, w):
        if w.has_lm_head or getattr(w, "has_embedding", False):
            raise ValueError("the scalar-loop tier covers middle stages only")
        return cls(w.block_kind, w.n_layers, w.d_model, w.n_heads, w.d_ffn, w.seq_len, w.microbatch, w.ln_eps)

    def forward(self, theta, x, valid_len=None):
        theta = np.ascontiguousarray(theta, dtype=np.float64)
        x = np.ascontiguousarray(x, dtype=np.float64)
        assert theta.size == self.n_params and x.shape == (self.N, self.D)
        y = np.empty((self.N, self.D))
        saved = np.empty(self.saved_doubles)
        vl = None if valid_len is None else np.ascontiguousarray(valid_len, dtype=np.int32)
        rc = lib().slow_stage_forward(*self.shape, self.eps, _ptr(theta), _ptr(x), None if vl is None else _ptr(vl),
                                      _ptr(y), _ptr(saved))
        if rc:
            raise MemoryError("slow_stage_forward")
        return y, saved

    def backward(self, theta, saved, dy):
        theta = np.ascontiguousarray(theta, dtype=np.float64)
        dy = np.ascontiguousarray(dy, dtype=np.float64)
        assert theta.size == self.n_params and dy.shape == (self.N, self.D) and saved.size == self.saved_doubles
        dx = np.empty((self.N, self.D))
        grad = np.empty(self.n_params)
        rc = lib().slow_stage_backward(*self.shape, self.eps, _ptr(theta), _ptr(saved), _ptr(dy), _ptr(dx), _ptr(grad))
        if rc:
            raise MemoryError("slow_stage_backward")
        return dx, grad
