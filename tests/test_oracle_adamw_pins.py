"""Pins of oracle/adamw_oracle.py (CPU only)."""
import numpy as np
import pytest

from oracle import adamw_oracle as O


def test_matches_the_library_optimizer_over_several_steps():
    """The algorithm the paper names (PPO hyperparameter table: AdamW, eps 1e-5, lr 3e-6) as the library
    implements it, in float64 on the CPU."""
    import torch
    g = np.random.default_rng(0)
    p0 = g.normal(0, 1, 257)
    for lr, wd in ((3e-6, 0.01), (1e-2, 0.0), (1e-3, 0.1)):
        tp = torch.nn.Parameter(torch.tensor(p0, dtype=torch.float64))
        opt = torch.optim.AdamW([tp], lr=lr, eps=1e-5, betas=(0.9, 0.999), weight_decay=wd)
        p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
        for step in range(1, 8):
            grad = g.normal(0, 1, 257) * (10.0 ** g.integers(-3, 2))
            tp.grad = torch.tensor(grad, dtype=torch.float64)
            opt.step()
            p, m, v = O.adamw_step(p, grad, m, v, step, lr=lr, weight_decay=wd)
            np.testing.assert_allclose(p, tp.detach().numpy(), rtol=1e-13, atol=1e-15)


def test_first_step_closed_form_and_scale_invariance():
    """t = 1 from zero moments: m_hat = g, v_hat = g^2, so p moves by -lr * g / (|g| + eps)."""
    g = np.random.default_rng(1)
    p0, grad = g.normal(0, 1, 100), g.normal(0, 3, 100)
    p, m, v = O.adamw_step(p0, grad, np.zeros(100), np.zeros(100), 1, lr=3e-6, weight_decay=0.0)
    np.testing.assert_allclose(p, p0 - 3e-6 * grad / (np.abs(grad) + 1e-5), rtol=0, atol=1e-18)
    np.testing.assert_allclose(m, 0.1 * grad, rtol=1e-13)
    np.testing.assert_allclose(v, 0.001 * grad * grad, rtol=1e-13)
    # a common factor on the gradients is what grad_scale applies
    p2, m2, v2 = O.adamw_step(p0, grad / 7.0, np.zeros(100), np.zeros(100), 1, lr=3e-6, weight_decay=0.0, grad_scale=7.0)
    np.testing.assert_allclose(p2, p, rtol=0, atol=1e-18)
    np.testing.assert_allclose(m2, m, rtol=1e-13)


def test_zero_gradient_leaves_pure_decoupled_decay():
    p0 = np.linspace(-2, 2, 41)
    m0, v0 = np.zeros(41), np.zeros(41)
    p, m, v = O.adamw_step(p0, np.zeros(41), m0, v0, 5, lr=1e-3, weight_decay=0.1)
    np.testing.assert_allclose(p, p0 * (1 - 1e-4), rtol=1e-15)
    assert not m.any() and not v.any()


def test_defaults_are_the_papers():
    import inspect
    sig = inspect.signature(O.adamw_step)
    assert sig.parameters["lr"].default == 3e-6 and sig.parameters["eps"].default == 1e-5


def test_linear_schedule_end_points():
    """PPO hyperparameter table, "Scheduler: Linear"."""
    assert O.linear_lr(3e-6, 0, 100) == 3e-6
    assert O.linear_lr(3e-6, 50, 100) == pytest.approx(1.5e-6, rel=1e-15)
    assert O.linear_lr(3e-6, 99, 100) == pytest.approx(3e-8, rel=1e-12)
    assert O.linear_lr(3e-6, 100, 100) == 0.0
    with pytest.raises(ValueError):
        O.linear_lr(3e-6, 0, 0)
    with pytest.raises(ValueError):
        O.adamw_step([0.0], [0.0], [0.0], [0.0], 0)
