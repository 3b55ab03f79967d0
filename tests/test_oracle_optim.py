"""Pins for the momentum / weight-decay / step-decay oracle: a library optimiser, closed
forms and the schedule the paper states."""
import numpy as np
import pytest
import torch

from oracle import optim as OO
from oracle import step as OS
import synth


def test_matches_library_sgd_over_several_steps():
    rng = np.random.default_rng(0)
    n, steps = 57, 6
    theta0 = rng.standard_normal(n)
    grads = rng.standard_normal((steps, n))
    lr, mu, wd = 0.05, 0.9, 5e-4
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, weight_decay=wd)
    theta, v = theta0.copy(), np.zeros(n)
    for s in range(steps):
        opt.zero_grad()
        p.grad = torch.tensor(grads[s], dtype=torch.float64)
        opt.step()
        theta, v = OO.momentum_sgd_update(theta, v, grads[s], lr, mu, wd)
        np.testing.assert_allclose(theta, p.detach().numpy(), rtol=1e-13, atol=1e-15)


def test_zero_momentum_zero_decay_is_plain_sgd():
    rng = np.random.default_rng(1)
    theta, g = rng.standard_normal(33), rng.standard_normal(33)
    t2, v2 = OO.momentum_sgd_update(theta, np.zeros(33), g, 0.3, 0.0, 0.0)
    assert np.array_equal(t2, theta - 0.3 * g) and np.array_equal(v2, g)


def test_constant_gradient_closed_form():
    # v_n = g (1 - mu^n) / (1 - mu);  theta_n = theta_0 - lr g sum_{i=1..n} (1 - mu^i)/(1 - mu)
    g, mu, lr = np.array([2.0, -3.0]), 0.9, 0.01
    theta, v = np.array([1.0, 1.0]), np.zeros(2)
    for n in range(1, 21):
        theta, v = OO.momentum_sgd_update(theta, v, g, lr, mu, 0.0)
        np.testing.assert_allclose(v, g * (1 - mu ** n) / (1 - mu), rtol=1e-12)
        s = sum((1 - mu ** i) / (1 - mu) for i in range(1, n + 1))
        np.testing.assert_allclose(theta, 1.0 - lr * g * s, rtol=1e-12)


def test_decay_only_is_geometric():
    theta, v = np.array([4.0, -2.0]), np.zeros(2)
    for n in range(1, 11):
        theta, v = OO.momentum_sgd_update(theta, v, np.zeros(2), 0.1, 0.0, 5e-4)
        np.testing.assert_allclose(theta, np.array([4.0, -2.0]) * (1 - 0.1 * 5e-4) ** n, rtol=1e-13)


def test_weighted_step_uses_the_weighted_aggregate():
    # same g as the plain step of the step oracle; with mu = wd = 0 the same parameters too
    layers = synth.mlp([6, 5, 3])
    rng = np.random.default_rng(3)
    theta = synth.he_normal_params(layers, 1, False).astype(np.float64)
    x = rng.standard_normal((7, 6))
    y = rng.integers(0, 3, 7)
    off = [0, 2, 7]
    ref = OS.sgd_step(layers, theta, x, y, off, 0.2)
    t2, v2, g = OO.weighted_momentum_step(theta, np.zeros_like(theta), ref.worker_grads, [2, 5], 0.2, 0.0, 0.0)
    np.testing.assert_allclose(g, ref.grad, rtol=1e-14, atol=1e-16)
    np.testing.assert_allclose(t2, ref.params, rtol=1e-14, atol=1e-16)
    # a mistake in the weights (uniform instead of b_k / B) must show
    wrong = 0.5 * ref.worker_grads[0] + 0.5 * ref.worker_grads[1]
    assert np.abs(wrong - g).max() > 1e-6


def test_step_decay_matches_library_schedule_and_the_stated_schedule():
    # the ResNet18 schedule of the paper's hyperparameter list: 0.1, divided by 10 after 15, 30, 45 epochs
    want = {0: 0.1, 14: 0.1, 15: 0.01, 29: 0.01, 30: 0.001, 44: 0.001, 45: 0.0001, 60: 0.0001}
    for e, lr in want.items():
        assert OO.lr_step_decay(0.1, 0.1, (15, 30, 45), e) == pytest.approx(lr, rel=1e-12)
    # VGG11: 0.01 with decay-rate 0.2 at epochs 15, 25, 35
    assert OO.lr_step_decay(0.01, 0.2, (15, 25, 35), 36) == pytest.approx(0.01 * 0.2 ** 3, rel=1e-12)
    p = torch.nn.Parameter(torch.zeros(1))
    opt = torch.optim.SGD([p], lr=0.1)
    sched = torch.optim.lr_scheduler.MultiStepLR(opt, milestones=[15, 30, 45], gamma=0.1)
    for e in range(50):
        assert OO.lr_step_decay(0.1, 0.1, (15, 30, 45), e) == pytest.approx(opt.param_groups[0]["lr"], rel=1e-12)
        opt.step()
        sched.step()
