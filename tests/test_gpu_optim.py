"""GPU parity of the optimiser step (Sec. 5.1: Adam) against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2405_04416_amd import binding as B
import sys

from gpu_util import DEV, dev, host

pytestmark = pytest.mark.gpu


def say(msg):
    print("[case]", msg)
    sys.stdout.flush()


def _check(theta_d, m_d, v_d, theta, m, v, moved, m_scale, steps):
    # fp32 arithmetic against the double oracle: a few roundings per step.  Errors are measured against the sizes
    # of the terms that were added (`moved`: sum of the absolute updates so far; `m_scale`: the first-moment
    # recursion run on absolute gradients), since the sums themselves may cancel.
    assert np.all(np.abs(host(theta_d).astype(np.float64) - theta) <= steps * (2e-6 * moved + 1.3e-7 * np.abs(theta)) + 1e-30)
    assert np.all(np.abs(host(m_d).astype(np.float64) - m) <= steps * 1e-6 * m_scale + 1e-37)
    np.testing.assert_allclose(host(v_d), v, rtol=steps * 1e-6, atol=1e-37)


@pytest.mark.parametrize("n,skip,l2,half", [(100003, True, 0.0, False), (4096, False, 1e-6, True), (9411, False, 1e-6, True),
                                            (3, True, 0.0, False), (5, False, 0.0, True), (1 << 20, True, 0.0, False)])
def test_adam_step(n, skip, l2, half):
    say("adam n=%d skip=%s l2=%g half=%s" % (n, skip, l2, half))
    rng = np.random.default_rng(n)
    theta32 = (rng.standard_normal(n) * 0.1).astype(np.float32)
    theta, m, v = theta32.astype(np.float64), np.zeros(n), np.zeros(n)
    theta_d, m_d, v_d = dev(theta32), torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    half_d = torch.full((n,), 7.0, dtype=torch.float16, device=DEV) if half else None
    moved, m_scale = np.zeros(n), np.zeros(n)
    for step in range(1, 4):
        g32 = (rng.standard_normal(n) * 10.0 ** rng.integers(-7, 2, n)).astype(np.float32)
        if skip:
            g32[rng.random(n) < 0.6] = 0.0                       # most entries untouched, as in a big hash table
            if n > 1000:
                g32[200:900] = 0.0                               # whole wavefronts untouched
        g_d = dev(g32)
        lr = B.dg_cosine_lr(0.05, 0.005, step * 50000, 300000)
        B.dg_adam_step(theta_d, g_d, m_d, v_d, lr, step, l2=l2, skip_zero_grad=skip, param_half=half_d)
        f32 = lambda x: float(np.float32(x))                     # the boundary takes fp32 hyper-parameters: same values for the oracle
        was = theta.copy()
        oracle.adam_step(theta, g32.astype(np.float64), m, v, lr=f32(lr), step=step, beta1=f32(0.9), beta2=f32(0.99), eps=f32(1e-15),
                         l2=f32(l2), skip_zero=skip)
        moved += np.abs(theta - was)
        used = (g32 != 0.0) | (not skip)
        m_scale = np.where(used, 0.9 * m_scale + 0.1 * (np.abs(g32) + l2 * np.abs(was)), m_scale)
        assert torch.count_nonzero(g_d).item() == 0              # the gradient is consumed
        if skip:                                                 # untouched entries: bit-identical value and moments
            still = (g32 == 0.0)
            prev = theta32 if step == 1 else prev_theta
            assert np.array_equal(host(theta_d)[still], prev[still])
        prev_theta = host(theta_d).copy()
        _check(theta_d, m_d, v_d, theta, m, v, moved, m_scale, step)
    if half:
        got = host(half_d)
        np.testing.assert_array_equal(got, host(theta_d).astype(np.float16))     # the rounded new values, all of them (dense)


def test_adam_rejects_bad_arguments():
    x = torch.zeros(16, device=DEV)
    with pytest.raises(B.DistGridError):
        B.dg_adam_step(x, x.clone(), x.clone(), x.clone(), 0.01, 0)            # steps count from 1
    with pytest.raises(B.DistGridError):
        B.dg_adam_step(x, x.clone(), x.clone(), x.clone(), 0.01, 1, beta1=1.0)
    with pytest.raises(B.DistGridError):
        B.dg_adam_step(x[1:], x.clone()[1:], x.clone()[1:], x.clone()[1:], 0.01, 1)      # misaligned
