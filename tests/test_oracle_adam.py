"""Pins for the oracle's optimiser step (Sec. 5.1: Adam with a cosine learning-rate schedule).

The recursion is pinned to things other than itself: closed forms of Adam's first step and of a constant gradient,
a library implementation of the published algorithm (torch.optim.Adam on float64), its scale invariance, and the
skip rule for untouched entries.
"""
import numpy as np
import pytest
import torch

import oracle


def _state(n, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(n), np.zeros(n), np.zeros(n)


def test_first_step_moves_by_lr_times_sign():
    # t = 1: m_hat = g, v_hat = g^2, so the step is lr * g / (|g| + eps): lr * sign(g) for |g| >> eps
    theta, m, v = _state(1000, 0)
    before = theta.copy()
    g = np.random.default_rng(1).standard_normal(1000) * 10.0 ** np.random.default_rng(2).integers(-6, 3, 1000)
    oracle.adam_step(theta, g, m, v, lr=0.05, step=1)
    np.testing.assert_allclose(theta - before, -0.05 * g / (np.abs(g) + 1e-15), rtol=1e-9)
    big = np.abs(g) > 1e-3
    np.testing.assert_allclose((theta - before)[big], -0.05 * np.sign(g[big]), rtol=1e-9)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v, 0.01 * g * g, rtol=1e-12)


def test_constant_gradient_closed_form():
    # with the same gradient every step the bias-corrected moments are g and g^2 at every t
    theta, m, v = _state(64, 3)
    before = theta.copy()
    g = np.random.default_rng(4).standard_normal(64) * 3.0
    for t in range(1, 41):
        oracle.adam_step(theta, g, m, v, lr=0.01, step=t, eps=1e-3)
    np.testing.assert_allclose(theta - before, -40 * 0.01 * g / (np.abs(g) + 1e-3), rtol=1e-9)


@pytest.mark.parametrize("l2", [0.0, 1e-2])
def test_matches_library_adam(l2):
    rng = np.random.default_rng(5)
    theta, m, v = _state(257, 6)
    ref = torch.tensor(theta.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([ref], lr=0.05, betas=(0.9, 0.99), eps=1e-15, weight_decay=l2)
    for t in range(1, 26):
        g = rng.standard_normal(257) * rng.choice([1e-4, 1.0, 30.0], 257)
        ref.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        oracle.adam_step(theta, g, m, v, lr=0.05, step=t, l2=l2)
    np.testing.assert_allclose(theta, ref.detach().numpy(), rtol=1e-10, atol=1e-12)


def test_gradient_scale_invariance():
    # moments scale as c and c^2, so the step does not change (eps far below |g|)
    rng = np.random.default_rng(7)
    a, ma, va = _state(100, 8)
    b, mb, vb = a.copy(), ma.copy(), va.copy()
    for t in range(1, 11):
        g = rng.standard_normal(100)
        oracle.adam_step(a, g, ma, va, lr=0.02, step=t)
        oracle.adam_step(b, 1024.0 * g, mb, vb, lr=0.02, step=t)
    np.testing.assert_allclose(a, b, rtol=1e-9)
    np.testing.assert_allclose(mb, 1024.0 * ma, rtol=1e-12)


def test_untouched_entries_are_left_alone():
    rng = np.random.default_rng(9)
    theta, m, v = _state(200, 10)
    oracle.adam_step(theta, rng.standard_normal(200), m, v, lr=0.05, step=1, skip_zero=True)     # every moment non-zero now
    g = rng.standard_normal(200)
    g[::3] = 0.0
    t0, m0, v0 = theta.copy(), m.copy(), v.copy()
    oracle.adam_step(theta, g, m, v, lr=0.05, step=2, skip_zero=True)
    hit = g != 0.0
    assert np.array_equal(theta[~hit], t0[~hit]) and np.array_equal(m[~hit], m0[~hit]) and np.array_equal(v[~hit], v0[~hit])
    assert np.all(theta[hit] != t0[hit])
    # without the rule the same entries keep moving on their momentum
    t1, m1, v1 = t0.copy(), m0.copy(), v0.copy()
    oracle.adam_step(t1, g, m1, v1, lr=0.05, step=2, skip_zero=False)
    assert np.all(t1[~hit] != t0[~hit])
    np.testing.assert_array_equal(t1[hit], theta[hit])


def test_cosine_schedule_of_the_paper():
    # Sec. 5.1: 0.05 down to 0.005 over 300k iterations
    assert oracle.cosine_lr(0.05, 0.005, 0, 300000) == pytest.approx(0.05, rel=1e-15)
    assert oracle.cosine_lr(0.05, 0.005, 300000, 300000) == pytest.approx(0.005, rel=1e-15)
    assert oracle.cosine_lr(0.05, 0.005, 150000, 300000) == pytest.approx(0.0275, rel=1e-12)
    assert oracle.cosine_lr(0.05, 0.005, 100000, 300000) == pytest.approx(0.005 + 0.045 * 0.75, rel=1e-12)     # cos(pi/3) = 1/2
    assert oracle.cosine_lr(0.05, 0.005, 400000, 300000) == pytest.approx(0.005, rel=1e-15)
    lrs = [oracle.cosine_lr(0.05, 0.005, i, 1000) for i in range(1001)]
    assert all(a > b for a, b in zip(lrs, lrs[1:]))
