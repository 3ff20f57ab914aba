"""Pins of the optimizer oracle (oracle/adamw_oracle.py) against things other
than itself: torch's own AdamW run in float64, and closed forms that follow from
the update rule (Adam with decoupled weight decay; the paper, Sec. 4, only names
the optimizer)."""
import numpy as np
import torch

from oracle import adamw_oracle as A


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_matches_an_independent_library_implementation_over_several_steps():
    theta = _rand((37, 5), 0)
    m = np.zeros_like(theta)
    v = np.zeros_like(theta)
    p = torch.nn.Parameter(torch.from_numpy(theta.copy()))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.8, 0.95), eps=1e-6, weight_decay=0.1)
    for t in range(1, 8):
        g = _rand(theta.shape, 100 + t) * (10.0 ** (t % 3 - 1))
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        theta, m, v = A.adamw_step(theta, g, m, v, t, lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1)
        np.testing.assert_allclose(theta, p.detach().numpy(), rtol=1e-12, atol=1e-14)
    st = opt.state[p]
    np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-15)


def test_first_step_from_zero_moments_has_a_closed_form():
    theta, g = _rand(1000, 1), _rand(1000, 2)
    lr, eps, wd = 1e-2, 1e-3, 0.05
    out, m, v = A.adamw_step(theta, g, 0 * g, 0 * g, 1, lr=lr, beta1=0.9, beta2=0.999, eps=eps, weight_decay=wd)
    np.testing.assert_allclose(out, theta - lr * (g / (np.abs(g) + eps) + wd * theta), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-13)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-12)


def test_zero_gradient_is_pure_decay_and_keeps_zero_moments():
    theta = _rand(64, 3)
    out, m, v = A.adamw_step(theta, 0 * theta, 0 * theta, 0 * theta, 4, lr=0.1, weight_decay=0.2, eps=1e-8)
    np.testing.assert_allclose(out, theta * (1 - 0.1 * 0.2), rtol=1e-14)
    assert not m.any() and not v.any()


def test_constant_gradient_moves_every_coordinate_by_lr_per_step():
    # with a constant gradient the bias-corrected moments are g and g*g at every step
    theta0, g = _rand(50, 4), _rand(50, 5)
    theta, m, v = theta0, 0 * g, 0 * g
    T, lr, eps = 25, 1e-3, 1e-9
    for t in range(1, T + 1):
        theta, m, v = A.adamw_step(theta, g, m, v, t, lr=lr, beta1=0.9, beta2=0.99, eps=eps, weight_decay=0.0)
    np.testing.assert_allclose(theta, theta0 - T * lr * g / (np.abs(g) + eps), rtol=1e-10, atol=1e-13)


def test_update_does_not_depend_on_the_gradient_scale_without_eps():
    theta = _rand(40, 6)
    gs = [_rand(40, 10 + t) for t in range(4)]
    res = []
    for c in (1.0, 1e3):
        th, m, v = theta, 0 * theta, 0 * theta
        for t, g in enumerate(gs, 1):
            th, m, v = A.adamw_step(th, c * g, m, v, t, lr=1e-2, eps=0.0, weight_decay=0.0)
        res.append(th)
    np.testing.assert_allclose(res[0], res[1], rtol=1e-12)


def test_bias_correction_uses_the_step_counter():
    # same moments, later step: a smaller correction, hence a smaller move (would not show if t were ignored)
    theta, g = np.ones(8), np.full(8, 0.5)
    a, _, _ = A.adamw_step(theta, g, 0 * g, 0 * g, 1, lr=0.1, weight_decay=0.0, eps=0.0)
    b, _, _ = A.adamw_step(theta, g, 0 * g, 0 * g, 10, lr=0.1, weight_decay=0.0, eps=0.0)
    np.testing.assert_allclose(theta - a, 0.1)
    expect = 0.1 * (0.1 * 0.5 / (1 - 0.9 ** 10)) / np.sqrt(0.001 * 0.25 / (1 - 0.999 ** 10))
    np.testing.assert_allclose(theta - b, expect, rtol=1e-12)


def test_sgd_step():
    np.testing.assert_allclose(A.sgd_step(np.array([1.0, -2.0]), np.array([0.5, 4.0]), 0.1), [0.95, -2.4])
