"""The oracle's two tiers against each other (no GPU): the numpy tier
(oracle/stage.py) and the scalar-loop C tier (oracle/slow_stage.c) are written
separately from the same textbook definitions, so a dropped term, a wrong
index or a transposed operand in either one shows as a difference far above
the rounding-order noise of double precision."""
import numpy as np
import pytest

import workloads as W
from oracle.slow import SlowStage
from oracle.stage import Stage


def _inputs(w, mb):
    st = Stage.from_workload(w)
    theta = W.make_theta(w, st.layout).astype(np.float64)
    x = W.make_x(w, mb).astype(np.float64)
    dy = W.make_dy(w, mb).astype(np.float64)
    valid = W.make_valid_len(w, mb) if w.block_kind == W.configs.BERT_POSTLN_BIDIR else None
    return st, theta, x, dy, valid


def _close(a, b, what, tol=1e-11):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    scale = max(np.abs(b).max(), 1e-300)
    err = np.abs(a - b).max() / scale
    assert err <= tol, (what, float(err))


CASES = [W.TINY["gpt"].with_(stage=1), W.TINY["bert"], W.TINY["gpt_mid"].with_(seq_len=72), W.TINY["bert_mid"].with_(seq_len=56),
         W.CONFIGS[1]]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_scalar_loops_match_numpy_tier(w):
    st, theta, x, dy, valid = _inputs(w, 0)
    slow = SlowStage.from_workload(w)
    assert slow.n_params == st.n_params
    y_ref, saved_ref = st.forward(theta, x, valid)
    dx_ref, g_ref = st.backward(theta, saved_ref, dy)
    y, saved = slow.forward(theta, x, valid)
    dx, g = slow.backward(theta, saved, dy)
    _close(y, y_ref, "Y")
    _close(dx, dx_ref, "dX")
    _close(g, g_ref, "flat gradient")
    # slice by slice: a small tensor (a bias, a LayerNorm gain) must not hide under a large one
    for name, off, r, c in st.layout:
        _close(g[off:off + r * c], g_ref[off:off + r * c], name, tol=1e-10)


@pytest.mark.parametrize("key", ["gpt", "bert"])
def test_backward_with_another_version(key):
    """Activations of the forward's version, parameters of another (Section 3.1's
    backward with the current weights): both tiers take the parameters from the
    vector handed to backward and everything else from what forward saved."""
    w = W.TINY[key].with_(stage=1)
    st, theta, x, dy, valid = _inputs(w, 1)
    rng = np.random.default_rng(5)
    theta_b = theta + 0.05 * rng.standard_normal(theta.size)
    slow = SlowStage.from_workload(w)
    _, saved_ref = st.forward(theta, x, valid)
    dx_ref, g_ref = st.backward(theta_b, saved_ref, dy)
    _, saved = slow.forward(theta, x, valid)
    dx, g = slow.backward(theta_b, saved, dy)
    _close(dx, dx_ref, "dX")
    _close(g, g_ref, "flat gradient")
    dx_same, _ = slow.backward(theta, saved, dy)
    assert np.abs(dx_same - dx).max() > 1e-6 * np.abs(dx).max()      # the version does enter


def test_middle_stages_only():
    with pytest.raises(ValueError):
        SlowStage.from_workload(W.TINY["lmhead"])
    with pytest.raises(ValueError):
        SlowStage.from_workload(W.TINY["embed"])
