"""Pins for oracle/optim.py (no GPU)."""
import numpy as np
import torch

from oracle import optim


def test_first_step_closed_form():
    rng = np.random.default_rng(0)
    th = rng.standard_normal(1000)
    g = rng.standard_normal(1000) * 1e-3
    lr, eps = 1e-4, 1e-8
    th2, m, v = optim.adam_step(th, np.zeros(1000), np.zeros(1000), g, 1, lr, 0.9, 0.999, eps)
    assert np.allclose(th2 - th, -lr * g / (np.abs(g) + eps), rtol=1e-9, atol=0)  # th ~ 1: the difference keeps ~12 digits
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)


def test_constant_gradient_limit():
    th = np.zeros(4)
    m = np.zeros(4)
    v = np.zeros(4)
    g = np.array([2.0, -3.0, 0.5, -1e-3])
    for t in range(1, 200):
        th_new, m, v = optim.adam_step(th, m, v, g, t, 1e-3, 0.9, 0.999, 1e-12)
        assert np.allclose(th_new - th, -1e-3 * np.sign(g), rtol=1e-6)
        th = th_new


def test_against_torch_adam_and_adamw():
    rng = np.random.default_rng(3)
    th0 = rng.standard_normal(257)
    grads = [rng.standard_normal(257) * 10.0 ** rng.integers(-4, 1) for _ in range(5)]
    for wd, cls in ((0.0, torch.optim.Adam), (0.1, torch.optim.AdamW)):
        p = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
        opt = cls([p], lr=3e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=wd)
        th, m, v = th0.copy(), np.zeros(257), np.zeros(257)
        for t, g in enumerate(grads, 1):
            p.grad = torch.tensor(g)
            opt.step()
            th, m, v = optim.adam_step(th, m, v, g, t, 3e-3, 0.9, 0.999, 1e-8, weight_decay=wd)
            # torch puts eps after dividing sqrt(v) by sqrt(1-b2^t): identical algebra
            assert np.allclose(th, p.detach().numpy(), rtol=1e-11, atol=1e-13)


def test_appendix_form_without_bias_correction():
    # Appendix B.1 as printed: m, v moving averages, P = 1/(sqrt(v)+eps), theta -= eta P m
    rng = np.random.default_rng(4)
    th, m, v, g = (rng.standard_normal(64) for _ in range(4))
    v = np.abs(v)
    th2, m2, v2 = optim.adam_step(th, m, v, g, 7, 1e-2, 0.9, 0.99, 1e-6, bias_correction=False)
    m_ref = 0.9 * m + 0.1 * g
    v_ref = 0.99 * v + 0.01 * g ** 2
    assert np.allclose(m2, m_ref, rtol=1e-13, atol=0) and np.allclose(v2, v_ref, rtol=1e-13, atol=0)
    assert np.allclose(th2, th - 1e-2 * m_ref / (np.sqrt(v_ref) + 1e-6), rtol=1e-12)


def test_grad_scale_is_mean():
    rng = np.random.default_rng(5)
    th, G = rng.standard_normal(32), rng.standard_normal(32)
    a = optim.adam_step(th, np.zeros(32), np.zeros(32), G, 1, 1e-3, 0.9, 0.999, 1e-8, grad_scale=0.125)
    b = optim.adam_step(th, np.zeros(32), np.zeros(32), G / 8, 1, 1e-3, 0.9, 0.999, 1e-8)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_accumulate_is_a_sum():
    rng = np.random.default_rng(6)
    gs = [rng.standard_normal(100) for _ in range(7)]
    G = np.zeros(100)
    for g in gs:
        optim.accumulate(G, g)
    ref = np.zeros(100)
    for g in gs:
        ref = ref + g
    assert np.array_equal(G, ref)


def test_bf16_rounding_matches_torch_cast():
    # every exponent, a sweep of mantissa patterns including exact ties
    hi = np.arange(0, 1 << 16, 7, dtype=np.uint32) << 16
    lows = np.array([0, 1, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x1234, 0xC000], dtype=np.uint32)
    bits = (hi[:, None] | lows[None, :]).reshape(-1)
    f = bits.view(np.float32)
    f = f[np.isfinite(f)]
    mine = optim.round_to_bf16(f)
    ref = torch.tensor(f).to(torch.bfloat16).to(torch.float64).numpy()
    keep = np.isfinite(ref)       # values that round up to infinity are outside the weights' range
    assert np.array_equal(mine[keep], ref[keep])
