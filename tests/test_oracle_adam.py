"""Pins of the optimiser oracle (App. B): none of them re-types its formula."""
import math

import numpy as np
import pytest
import torch

from oracle import adam as A


def test_lr_schedule_values_from_the_configuration_table():
    # App. B: 1024^-0.5 * min(step^-0.5, step * 4000^-1.5)
    peak = A.lr_schedule(4000, 1024, 4000)
    assert math.isclose(peak, 1.0 / (32.0 * math.sqrt(4000.0)), rel_tol=1e-15)        # both branches meet
    assert math.isclose(A.lr_schedule(1, 1024, 4000), 1.0 / 32.0 / 4000.0 ** 1.5, rel_tol=1e-15)
    assert math.isclose(A.lr_schedule(16000, 1024, 4000), peak / 2.0, rel_tol=1e-15)  # 4x steps -> half
    assert math.isclose(A.lr_schedule(2000, 1024, 4000), peak / 2.0, rel_tol=1e-15)   # linear warm-up
    xs = [A.lr_schedule(s) for s in range(1, 9000)]
    assert int(np.argmax(xs)) + 1 == 4000
    with pytest.raises(ValueError):
        A.lr_schedule(0)


def test_first_step_closed_form():
    """From zero moments the bias-corrected moments are g and g^2: the step is lr * g / (|g| + eps)."""
    rng = np.random.default_rng(0)
    th, g = rng.normal(size=100), rng.normal(size=100) * 1e-3
    new, m, v = A.adam_step(th, g, np.zeros(100), np.zeros(100), 1, 0.01)
    np.testing.assert_allclose(new, th - 0.01 * g / (np.abs(g) + A.EPS), rtol=1e-12, atol=0)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v, 0.02 * g * g, rtol=1e-12)


def test_against_torch_adam_over_several_steps():
    """An independent implementation (torch.optim.Adam, float64, CPU) fed the same gradients."""
    rng = np.random.default_rng(1)
    th0 = rng.normal(size=(7, 13)) * 0.02
    p = torch.nn.Parameter(torch.from_numpy(th0.copy()))
    opt = torch.optim.Adam([p], lr=1.0, betas=(A.BETA1, A.BETA2), eps=A.EPS)
    th, m, v = th0.copy(), np.zeros_like(th0), np.zeros_like(th0)
    for step in range(1, 8):
        g = rng.normal(size=th0.shape) * (10.0 ** rng.integers(-6, 1))
        lr = A.lr_schedule(step, 512, 10)
        for grp in opt.param_groups:
            grp["lr"] = lr
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        th, m, v = A.adam_step(th, g, m, v, step, lr)
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-11, atol=1e-15)


def test_gradient_scale_invariance():
    """Adam's step does not depend on the scale of the gradients (up to eps)."""
    rng = np.random.default_rng(2)
    th, g1, g2 = rng.normal(size=50), rng.normal(size=50), rng.normal(size=50)
    def two_steps(c):
        a, m, v = A.adam_step(th, c * g1, np.zeros(50), np.zeros(50), 1, 0.1, eps=0.0)
        return A.adam_step(a, c * g2, m, v, 2, 0.1, eps=0.0)[0]
    np.testing.assert_allclose(two_steps(1.0), two_steps(1000.0), rtol=1e-12)


def test_inputs_are_not_modified():
    th, g, m, v = np.ones(4), np.ones(4), np.ones(4), np.ones(4)
    A.adam_step(th, g, m, v, 3, 0.5)
    assert (th == 1).all() and (m == 1).all() and (v == 1).all()
