"""Pins for the oracle's optimiser formulas: hand-computed steps, first-step
closed forms and torch.optim in float64 (a library cross-check)."""
import math
import numpy as np
import torch

from oracle import optim


def test_sgd_momentum_hand_computed():
    th = np.array([1.0, -2.0, 0.5])
    v = np.zeros(3)
    g1 = np.array([0.5, -1.0, 2.0])
    th, v = optim.sgd_momentum(th, g1, v, np.float32(0.1), 0.9)
    lr = float(np.float32(0.1))
    assert np.allclose(th, [1.0 - lr * 0.5, -2.0 + lr * 1.0, 0.5 - lr * 2.0], atol=1e-15)
    g2 = np.array([1.0, 1.0, -1.0])
    th, v = optim.sgd_momentum(th, g2, v, np.float32(0.1), 0.9)
    # v2 = 0.9 g1 + g2
    assert np.allclose(v, [1.45, 0.1, 0.8], atol=1e-15)
    assert np.allclose(th, [1.0 - lr * (0.5 + 1.45), -2.0 - lr * (-1.0 + 0.1), 0.5 - lr * (2.0 + 0.8)], atol=1e-14)


def test_adam_first_step_closed_form():
    # from zero state: mhat = g, vhat = g^2 -> step = -lr (g/(|g|+eps) + wd theta)
    th = np.array([1.0, -2.0, 0.5])
    g = np.array([0.3, -4.0, 1e-3])
    lr, b1, wd = np.float32(0.01), np.float32(0.85), np.float32(1e-3)
    out, m, v = optim.adam(th, g, np.zeros(3), np.zeros(3), 1, lr, b1, 0.999, 1e-8, wd)
    ref = th - float(lr) * (g / (np.abs(g) + 1e-8) + float(wd) * th)
    assert np.allclose(out, ref, rtol=0, atol=1e-15)
    assert np.allclose(m, (1 - float(b1)) * g) and np.allclose(v, 0.001 * g * g)


def test_adam_second_step_hand_computed():
    b1, b2, eps, lr = 0.5, 0.999, 1e-8, 0.125
    th, m, v = np.array([2.0]), np.zeros(1), np.zeros(1)
    th, m, v = optim.adam(th, np.array([1.0]), m, v, 1, lr, b1, b2, eps, 0.0)
    th, m, v = optim.adam(th, np.array([3.0]), m, v, 2, lr, b1, b2, eps, 0.0)
    m2 = 0.5 * 0.5 + 0.5 * 3.0                      # 1.75
    v2 = 0.999 * 0.001 + 0.001 * 9.0
    step2 = lr * (m2 / 0.75) / (math.sqrt(v2 / (1 - 0.999 ** 2)) + eps)
    step1 = lr * 1.0 / (1.0 + eps)
    assert abs(th[0] - (2.0 - step1 - step2)) < 1e-15


def test_rmsprop_first_step_closed_form():
    th = np.array([1.0, -1.0])
    g = np.array([0.2, -3.0])
    out, s = optim.rmsprop(th, g, np.zeros(2), np.float32(1e-3), 0.99, 1e-5)
    ref = th - float(np.float32(1e-3)) * g / np.sqrt(0.01 * g * g + 1e-5)
    assert np.allclose(out, ref, atol=1e-16)
    out2, s2 = optim.rmsprop(out, g, s, np.float32(1e-3), 0.99, 1e-5)
    assert np.allclose(s2, 0.99 * 0.01 * g * g + 0.01 * g * g)


def _torch_run(opt_cls, kwargs, th0, grads):
    p = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    opt = opt_cls([p], **kwargs)
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    return p.detach().numpy()


def test_against_torch_optimizers():
    rng = np.random.default_rng(0)
    th0 = rng.standard_normal(16)
    grads = [rng.standard_normal(16) for _ in range(6)]
    lr = float(np.float32(0.02))

    th, v = th0.copy(), np.zeros(16)
    for g in grads:
        th, v = optim.sgd_momentum(th, g, v, np.float32(0.02), 0.9)
    assert np.allclose(th, _torch_run(torch.optim.SGD, dict(lr=lr, momentum=0.9), th0, grads), atol=1e-13)

    th, m, v = th0.copy(), np.zeros(16), np.zeros(16)
    b1, wd = float(np.float32(0.87)), float(np.float32(3e-3))
    for t, g in enumerate(grads, 1):
        th, m, v = optim.adam(th, g, m, v, t, np.float32(0.02), np.float32(0.87), 0.999, 1e-8, np.float32(3e-3))
    ref = _torch_run(torch.optim.AdamW, dict(lr=lr, betas=(b1, 0.999), eps=1e-8, weight_decay=wd), th0, grads)
    assert np.allclose(th, ref, atol=1e-12)

    # torch's RMSprop puts eps outside the square root; the two agree at eps = 0
    th, s = th0.copy(), np.zeros(16)
    for g in grads:
        th, s = optim.rmsprop(th, g, s, np.float32(0.02), 0.99, 0.0)
    ref = _torch_run(torch.optim.RMSprop, dict(lr=lr, alpha=0.99, eps=0.0), th0, grads)
    assert np.allclose(th, ref, atol=1e-12)
