"""Pins for the oracle's network arithmetic: central finite differences, closed
forms and a library cross-check (torch autograd in float64)."""
import math
import numpy as np
import pytest
import torch

from oracle import nets


def _rand_params(dims, rng):
    return [(rng.standard_normal((a, b)) * 0.7, rng.standard_normal(b) * 0.3)
            for a, b in zip(dims[:-1], dims[1:])]


@pytest.mark.parametrize("kind", [nets.ACT_RELU, nets.ACT_GELU, nets.ACT_LEAKY_RELU, nets.ACT_TANH])
def test_activation_derivative_fd(kind):
    z = np.linspace(-3.1, 2.9, 41) + 0.013          # never exactly 0
    e = 1e-6
    fd = (nets.act(z + e, kind) - nets.act(z - e, kind)) / (2 * e)
    assert np.allclose(fd, nets.act_grad(z, kind), atol=1e-8)


def test_activation_values():
    z = np.array([-2.0, -0.5, 0.0, 0.5, 2.0])
    assert np.allclose(nets.act(z, nets.ACT_RELU), [0, 0, 0, 0.5, 2])
    assert np.allclose(nets.act(z, nets.ACT_LEAKY_RELU), [-0.4, -0.1, 0, 0.5, 2])
    # GELU(z) = z * Phi(z), Phi from math.erfc independently
    ref = [v * 0.5 * math.erfc(-v / math.sqrt(2)) for v in z]
    assert np.allclose(nets.act(z, nets.ACT_GELU), ref, atol=1e-15)
    assert np.allclose(nets.act(z, nets.ACT_TANH), [math.tanh(v) for v in z])


@pytest.mark.parametrize("kind", [nets.ACT_RELU, nets.ACT_GELU, nets.ACT_LEAKY_RELU, nets.ACT_TANH])
def test_classifier_gradients_fd(kind):
    rng = np.random.default_rng(3)
    dims = [3, 5, 4, 2]
    params = _rand_params(dims, rng)
    x = rng.standard_normal((6, 3))
    y = rng.integers(0, 2, size=6)
    loss, grads = nets.classifier_loss_and_grads(params, x, y, kind)
    e = 1e-6
    for l in range(len(params)):
        for which in (0, 1):
            arr = params[l][which]
            g = grads[l][which]
            it = np.nditer(arr, flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = arr[idx]
                arr[idx] = old + e
                lp = nets.classifier_loss_and_grads(params, x, y, kind)[0]
                arr[idx] = old - e
                lm = nets.classifier_loss_and_grads(params, x, y, kind)[0]
                arr[idx] = old
                assert abs((lp - lm) / (2 * e) - g[idx]) <= 1e-6 * max(1.0, abs(g[idx]))


def test_input_gradient_fd():
    rng = np.random.default_rng(5)
    params = _rand_params([4, 6, 3], rng)
    x = rng.standard_normal((2, 4))
    w = rng.standard_normal((2, 3))
    out, cache = nets.mlp_forward(params, x, nets.ACT_TANH, nets.ACT_TANH)
    _, dx = nets.mlp_backward(params, cache, w, nets.ACT_TANH, nets.ACT_TANH)
    e = 1e-6
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += e
        xm[idx] -= e
        fp = (nets.mlp_forward(params, xp, nets.ACT_TANH, nets.ACT_TANH)[0] * w).sum()
        fm = (nets.mlp_forward(params, xm, nets.ACT_TANH, nets.ACT_TANH)[0] * w).sum()
        assert abs((fp - fm) / (2 * e) - dx[idx]) < 1e-7


@pytest.mark.parametrize("smoothing", [0.0, 0.1, 0.35])
def test_xent_uniform_logits_closed_form(smoothing):
    # At equal logits every class has probability 1/C, so the loss is ln C for
    # any target distribution, and the gradient is (1/C - q)/n.
    C, n = 7, 5
    logits = np.full((n, C), 3.25)
    labels = np.arange(n) % C
    loss, d = nets.softmax_xent(logits, labels, smoothing)
    assert abs(loss - math.log(C)) < 1e-14
    assert np.allclose(d.sum(axis=1), 0.0, atol=1e-16)
    assert np.isclose(d[0, labels[0]], (1.0 / C - (1 - smoothing) - smoothing / C) / n)


def test_xent_matches_definition_and_shift_invariance():
    rng = np.random.default_rng(11)
    logits = rng.standard_normal((4, 5)) * 4
    labels = np.array([0, 4, 2, 2])
    loss, _ = nets.softmax_xent(logits, labels)
    ref = 0.0
    for i in range(4):
        p = [math.exp(v) for v in logits[i]]
        ref -= math.log(p[labels[i]] / sum(p))
    assert abs(loss - ref / 4) < 1e-13
    loss2, _ = nets.softmax_xent(logits + 1000.0, labels)
    assert abs(loss2 - loss) < 1e-10
    assert np.allclose(np.exp(nets.log_softmax(logits)).sum(axis=1), 1.0)


@pytest.mark.parametrize("kind,tkind", [(nets.ACT_RELU, "relu"), (nets.ACT_GELU, "gelu")])
def test_against_torch_autograd(kind, tkind):
    rng = np.random.default_rng(17)
    dims = [8, 16, 12, 5]
    params = _rand_params(dims, rng)
    x = rng.standard_normal((9, 8))
    y = rng.integers(0, 5, size=9)
    loss, grads = nets.classifier_loss_and_grads(params, x, y, kind)
    tp = [(torch.tensor(W, requires_grad=True), torch.tensor(b, requires_grad=True)) for W, b in params]
    a = torch.tensor(x)
    for l, (W, b) in enumerate(tp):
        a = a @ W + b
        if l < len(tp) - 1:
            a = torch.relu(a) if tkind == "relu" else torch.nn.functional.gelu(a)
    tl = torch.nn.functional.cross_entropy(a, torch.tensor(y, dtype=torch.long))
    tl.backward()
    assert abs(float(tl.detach()) - loss) < 1e-12
    for (W, b), (gW, gb) in zip(tp, grads):
        assert np.allclose(W.grad.numpy(), gW, atol=1e-12)
        assert np.allclose(b.grad.numpy(), gb, atol=1e-12)


def test_round_bf16_against_library_and_by_hand():
    rng = np.random.default_rng(23)
    x = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000), [0.0, -0.0, 1.0, -1.0]])
    x32 = x.astype(np.float32)          # exactly representable inputs, so one rounding on both sides
    ref = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(nets.round_bf16(x32.astype(np.float64)), ref)
    # spacing at 1.0 is 2**-7: ties go to the even neighbour
    assert nets.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert nets.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert nets.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -30]))[0] == 1.0 + 2.0 ** -7
    assert nets.round_bf16(np.array([-3.14159]))[0] == -3.140625


def test_bf16_storage_is_a_small_perturbation_of_the_exact_gradient():
    rng = np.random.default_rng(29)
    params = _rand_params([16, 32, 24, 5], rng)
    x = rng.standard_normal((20, 16))
    y = rng.integers(0, 5, size=20)
    l0, g0 = nets.classifier_loss_and_grads(params, x, y, nets.ACT_GELU)
    l1, g1 = nets.classifier_loss_and_grads(params, x, y, nets.ACT_GELU, q=nets.round_bf16)
    assert 0 < abs(l1 - l0) < 2e-2 * abs(l0)
    for (a, b), (c, d) in zip(g0, g1):
        assert 0 < np.linalg.norm(a - c) < 2e-2 * np.linalg.norm(a)
        assert np.linalg.norm(b - d) < 2e-2 * np.linalg.norm(b)
