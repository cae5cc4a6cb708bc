"""Oracle: gradient accumulation over a window and the Adam update.

TEST INFRASTRUCTURE ONLY (see the package docstring).

Section 3.3: gradients of the T minibatches of a window are summed and applied
in one update. Appendix B.1 gives the Adam-type rule: first and second moment
estimates m, v, a diagonal preconditioner 1/(sqrt(v)+eps) and the step
theta <- theta - eta * P * m. The appendix prints the rule without bias
correction; Section 4.1 names AdamW, whose standard form divides the moments
by (1 - beta^t) and adds a decoupled weight-decay term. Both are here: the
appendix form is `bias_correction=False, weight_decay=0`.
"""
import numpy as np


def accumulate(G, g):
    """G <- G + g (the window's running sum)."""
    G += g
    return G


def adam_step(theta, m, v, G, step, lr, beta1, beta2, eps, weight_decay=0.0,
              grad_scale=1.0, bias_correction=True):
    """One update, `step` counted from 1. Returns new (theta, m, v); inputs are
    not modified. eps sits outside the square root, as printed."""
    ghat = grad_scale * G
    m2 = beta1 * m + (1.0 - beta1) * ghat
    v2 = beta2 * v + (1.0 - beta2) * ghat * ghat
    if bias_correction:
        mh = m2 / (1.0 - beta1 ** step)
        vh = v2 / (1.0 - beta2 ** step)
    else:
        mh, vh = m2, v2
    theta2 = theta - lr * (mh / (np.sqrt(vh) + eps) + weight_decay * theta)
    return theta2, m2, v2


def round_to_bf16(a):
    """Nearest bfloat16 (ties to even) of each value, returned as float64.
    The input is first brought to float32, the precision the master weights
    are kept in."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    keep = bits >> 16
    rest = bits & 0xFFFF
    up = (rest > 0x8000) | ((rest == 0x8000) & ((keep & 1) == 1))
    keep = keep + up.astype(np.uint64)
    out = (keep << 16).astype(np.uint32).view(np.float32)
    return out.astype(np.float64).reshape(f.shape)


def round_to_fp32(a):
    return np.asarray(a, dtype=np.float32).astype(np.float64)
