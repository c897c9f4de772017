"""Pins for the oracle's GAN workload: closed forms, finite differences through both networks,
brute-force MMD, library cross-check of the logistic loss."""
import math
import numpy as np
import torch

from oracle import gan, nets, philox


def _spec(bf16=False):
    return gan.GanSpec([3, 6, 5], [5, 7, 4, 1], batch=4, seed=9, bf16_storage=bf16)


def _member(spec, rng, h=(1e-3, 2e-3)):
    mk = lambda dims: [(rng.standard_normal((a, b)) * 0.6, rng.standard_normal(b) * 0.2) for a, b in zip(dims[:-1], dims[1:])]
    return gan.new_member(spec, mk(spec.g_dims), mk(spec.d_dims), h, 0)


def test_softplus_sigmoid_logistic_closed_forms():
    x = np.array([-800.0, -3.0, 0.0, 2.5, 800.0])
    assert np.allclose(nets.softplus(x), [0.0, math.log1p(math.exp(-3.0)), math.log(2.0), 2.5 + math.log1p(math.exp(-2.5)), 800.0])
    assert np.allclose(nets.sigmoid(x), [0.0, 1 / (1 + math.exp(3.0)), 0.5, 1 / (1 + math.exp(-2.5)), 1.0])
    # at logit 0 the loss is ln 2 for any target and the gradient is (0.5 - t)/n
    loss, d = nets.logistic_loss(np.zeros((6, 1)), [1, 0, 1, 1, 0, 0])
    assert abs(loss - math.log(2.0)) < 1e-15 and np.allclose(d.ravel(), (0.5 - np.array([1, 0, 1, 1, 0, 0])) / 6)
    rng = np.random.default_rng(0)
    l, t = rng.standard_normal(9) * 3, rng.integers(0, 2, 9)
    ref = torch.nn.functional.binary_cross_entropy_with_logits(torch.tensor(l), torch.tensor(t, dtype=torch.float64))
    assert abs(nets.logistic_loss(l, t)[0] - float(ref)) < 1e-14


def _fd_check(loss_fn, arrays, grads, idxs, eps=1e-6, tol=1e-6):
    flat_g = [a for gr in grads for a in gr]
    for arr, g in zip(arrays, flat_g):
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = arr[idx]
            arr[idx] = old + eps
            lp = loss_fn()
            arr[idx] = old - eps
            lm = loss_fn()
            arr[idx] = old
            assert abs((lp - lm) / (2 * eps) - g[idx]) <= tol * max(1.0, abs(g[idx])), (idx, g[idx])


def test_discriminator_and_generator_gradients_fd():
    spec = _spec()
    rng = np.random.default_rng(1)
    m = _member(spec, rng)
    real = rng.standard_normal((4, 5))
    z = rng.standard_normal((4, 3))
    loss_d, gd = gan.d_loss_and_grads(spec, m, real, z)
    n_g = 2 * spec.n_g
    _fd_check(lambda: gan.d_loss_and_grads(spec, m, real, z)[0], m.theta[n_g:], gd, None)
    loss_g, gg = gan.g_loss_and_grads(spec, m, z)
    _fd_check(lambda: gan.g_loss_and_grads(spec, m, z)[0], m.theta[:n_g], gg, None)
    # definitions written out row by row
    fake = nets.mlp_forward(gan.g_params(spec, m), z, spec.g_hidden, spec.g_out)[0]
    D = lambda x: nets.mlp_forward(gan.d_params(spec, m), x, spec.d_hidden)[0].ravel()
    ref_d = np.mean([math.log1p(math.exp(-v)) for v in D(real)]) + np.mean([math.log1p(math.exp(v)) for v in D(fake)])
    assert abs(loss_d - ref_d) < 1e-12
    assert abs(loss_g - np.mean([math.log1p(math.exp(-v)) for v in D(fake)])) < 1e-12
    assert np.all(np.abs(fake) < 1.0)                      # tanh output


def test_step_updates_d_then_g_with_their_own_rates():
    spec = _spec()
    rng = np.random.default_rng(2)
    train = rng.standard_normal((32, 5)).astype(np.float32)
    m = _member(spec, rng, h=(0.0, 1e-2))                   # generator frozen
    before = [a.copy() for a in m.theta]
    gan.step(spec, m, 0, 0, train)
    n_g = 2 * spec.n_g
    assert all(np.array_equal(a, b) for a, b in zip(m.theta[:n_g], before[:n_g]))
    assert all(not np.array_equal(a, b) for a, b in zip(m.theta[n_g:], before[n_g:]))
    # first Adam step moves every discriminator weight by lr (up to eps): |delta| = lr |g| / (|g| + eps)
    assert np.allclose(np.abs(m.theta[n_g] - before[n_g]), float(np.float32(1e-2)), rtol=1e-4)
    m2 = _member(spec, np.random.default_rng(2), h=(1e-2, 0.0))   # discriminator frozen
    b2 = [a.copy() for a in m2.theta]
    gan.step(spec, m2, 0, 0, train)
    assert all(np.array_equal(a, b) for a, b in zip(m2.theta[n_g:], b2[n_g:])) and m2.t == 1
    assert not np.array_equal(m2.theta[0], b2[0])


def test_generator_step_sees_the_updated_discriminator():
    spec = _spec()
    train = np.random.default_rng(3).standard_normal((32, 5)).astype(np.float32)
    a = _member(spec, np.random.default_rng(4), h=(1e-2, 5e-2))
    b = _member(spec, np.random.default_rng(4), h=(1e-2, 0.0))
    gan.step(spec, a, 0, 0, train)
    gan.step(spec, b, 0, 0, train)
    assert not np.array_equal(a.theta[0], b.theta[0])


def test_latents_counter_assignment_and_moments():
    z = gan.latents(5, 3, 2, 1, 4, 6)
    e = 13                                                    # row 2, column 1: block 3, pair 0, sine branch
    w = philox.philox4x32_10([3, 2, philox.DOMAIN_LATENT + 1, e // 4], [5, 0])
    u1, u2 = (int(w[0]) + 0.5) / 2**32, (int(w[1]) + 0.5) / 2**32
    assert abs(z[2, 1] - math.sqrt(-2 * math.log(u1)) * math.sin(2 * math.pi * u2)) < 1e-14
    e = 14                                                    # pair 1, cosine branch
    u1, u2 = (int(w[2]) + 0.5) / 2**32, (int(w[3]) + 0.5) / 2**32
    assert abs(z[2, 2] - math.sqrt(-2 * math.log(u1)) * math.cos(2 * math.pi * u2)) < 1e-14
    big = gan.latents(5, 0, 0, 0, 500, 40)
    assert abs(big.mean()) < 0.02 and abs(big.std() - 1) < 0.02
    assert not np.array_equal(gan.latents(5, 0, 0, 0, 4, 6), gan.latents(5, 0, 0, 1, 4, 6))


def test_mmd_bruteforce_and_invariants():
    rng = np.random.default_rng(6)
    x, y = rng.standard_normal((8, 5)), rng.standard_normal((8, 5)) + 0.7
    k = lambda a, b: math.exp(-sum((p - q) ** 2 for p, q in zip(a, b)) / (2 * 5))
    ref = (sum(k(a, b) for a in x for b in x) + sum(k(a, b) for a in y for b in y) - 2 * sum(k(a, b) for a in x for b in y)) / 64
    assert abs(gan.rbf_mmd2(x, y) - ref) < 1e-14
    assert abs(gan.rbf_mmd2(x, x)) < 1e-15                   # biased estimator: exactly zero on identical samples
    assert abs(gan.rbf_mmd2(x, y) - gan.rbf_mmd2(y, x)) < 1e-15 and gan.rbf_mmd2(x, y) > 0
    assert gan.rbf_mmd2(x, y + 3.0) > gan.rbf_mmd2(x, y)


def test_bf16_storage_perturbs_slightly():
    rng = np.random.default_rng(7)
    real, z = rng.standard_normal((4, 5)), rng.standard_normal((4, 3))
    a, b = _member(_spec(), np.random.default_rng(8)), _member(_spec(True), np.random.default_rng(8))
    la, ga = gan.g_loss_and_grads(_spec(), a, z)
    lb, gb = gan.g_loss_and_grads(_spec(True), b, z)
    assert 0 < abs(la - lb) < 3e-2 * abs(la)
    assert np.linalg.norm(ga[0][0] - gb[0][0]) < 5e-2 * np.linalg.norm(ga[0][0])
