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


# ---- WGAN-GP (Section 4.3.1: the paper's objective, 5 critic updates per generator update) -----------

def _wspec(K=2, bf16=False):
    return gan.GanSpec([3, 6, 5], [5, 7, 4, 1], batch=4, seed=9, bf16_storage=bf16, objective="wgan_gp", n_critic=K)


def test_gradient_penalty_of_a_linear_critic_closed_form():
    """D(x) = x.w + b: the input gradient is w for every row, penalty = gp_weight (|w| - 1)^2 and
    d penalty / d w = 2 gp_weight (|w| - 1) w / |w|, whatever the rows are."""
    spec = gan.GanSpec([2, 3], [3, 1], batch=4, seed=1, objective="wgan_gp")
    w = np.array([[0.6], [-1.2], [2.0]])
    D = [(w, np.array([0.3]))]
    x = np.random.default_rng(0).standard_normal((5, 3))
    out, g, _, _ = gan.critic_input_gradient(spec, D, x)
    assert np.allclose(g, np.tile(w.T, (5, 1))) and np.allclose(out, x @ w + 0.3)
    nw = math.sqrt(0.36 + 1.44 + 4.0)
    pen, grads = gan.gradient_penalty_and_grads(spec, D, x)
    assert abs(pen - 10.0 * (nw - 1.0) ** 2) < 1e-12
    assert np.allclose(grads[0][0], 2 * 10.0 * (nw - 1.0) * w / nw) and np.all(grads[0][1] == 0.0)


def test_critic_input_gradient_and_penalty_gradient_fd():
    spec = _wspec()
    rng = np.random.default_rng(2)
    m = _member(spec, rng)
    D = gan.d_params(spec, m)
    x = rng.standard_normal((4, 5))
    out, g, _, _ = gan.critic_input_gradient(spec, D, x)
    f = lambda xx: nets.mlp_forward(D, xx, spec.d_hidden)[0].ravel()
    for r in range(4):
        for k in range(5):
            e = np.zeros_like(x)
            e[r, k] = 1e-6
            assert abs((f(x + e)[r] - f(x - e)[r]) / 2e-6 - g[r, k]) < 1e-6
    pen, grads = gan.gradient_penalty_and_grads(spec, D, x)
    # the penalty written out from its definition, with the input gradient by the network's own backward pass
    def penalty():
        gg = gan.critic_input_gradient(spec, gan.d_params(spec, m), x)[1]
        return 10.0 * np.mean([(math.sqrt(float(row @ row)) - 1.0) ** 2 for row in gg])
    assert abs(pen - penalty()) < 1e-12
    n_g = 2 * spec.n_g
    _fd_check(penalty, m.theta[n_g:], grads, None, tol=2e-6)
    assert all(np.all(gb == 0.0) for _, gb in grads)                 # the input gradient does not depend on the biases


def test_wgan_gp_losses_and_gradients_fd():
    spec = _wspec()
    rng = np.random.default_rng(3)
    m = _member(spec, rng)
    real, z, eps = rng.standard_normal((4, 5)), rng.standard_normal((4, 3)), rng.random(4)
    loss_d, gd = gan.critic_loss_and_grads(spec, m, real, z, eps)
    n_g = 2 * spec.n_g
    _fd_check(lambda: gan.critic_loss_and_grads(spec, m, real, z, eps)[0], m.theta[n_g:], gd, None, tol=2e-6)
    loss_g, gg = gan.wgan_generator_loss_and_grads(spec, m, z)
    _fd_check(lambda: gan.wgan_generator_loss_and_grads(spec, m, z)[0], m.theta[:n_g], gg, None)
    # definitions written out
    fake = nets.mlp_forward(gan.g_params(spec, m), z, spec.g_hidden, spec.g_out)[0]
    D = lambda x: nets.mlp_forward(gan.d_params(spec, m), x, spec.d_hidden)[0].ravel()
    xhat = eps[:, None] * real + (1 - eps[:, None]) * fake
    pen = gan.gradient_penalty_and_grads(spec, gan.d_params(spec, m), xhat)[0]
    assert abs(loss_d - (D(fake).mean() - D(real).mean() + pen)) < 1e-12
    assert abs(loss_g + D(fake).mean()) < 1e-12
    # eps = 1 puts the penalty on the real rows, eps = 0 on the generated ones
    assert abs(gan.critic_loss_and_grads(spec, m, real, z, np.ones(4))[0]
               - (D(fake).mean() - D(real).mean() + gan.gradient_penalty_and_grads(spec, gan.d_params(spec, m), real)[0])) < 1e-12


def test_wgan_gp_step_schedule_counters_and_update_counts():
    """K critic updates then one generator update; critic update k of step s uses batch counters k B + r,
    latent sub-stream 3 + k and eps from domain 14; the critic's Adam has had K (t-1) + k + 1 updates."""
    K = 3
    spec = _wspec(K=K)
    rng = np.random.default_rng(4)
    train_x = rng.standard_normal((50, 5))
    m = _member(spec, rng)
    twin = _member(spec, np.random.default_rng(4 + 0))         # rebuilt below from m's arrays
    twin.theta = [a.copy() for a in m.theta]
    twin.h = m.h.copy()
    B, n_g = spec.batch, 2 * spec.n_g
    # eps and rows against single Philox calls
    e = gan.gp_eps(spec.seed, 5, 2, 1, B)
    for r in range(B):
        w = philox.philox4x32_10([5, 2, gan.DOMAIN_GP_EPS, 1 * B + r], [spec.seed, 0])
        assert e[r] == (int(w[0]) + 0.5) / 2 ** 32
    # two steps by the oracle; the same two steps assembled by hand from the pieces, critic state through torch's Adam
    d_t = [torch.tensor(a.copy(), dtype=torch.float64, requires_grad=True) for a in twin.theta[n_g:]]
    opt_d = torch.optim.Adam(d_t, lr=float(twin.h[1]), betas=(spec.beta1, spec.beta2), eps=spec.eps)
    g_t = [torch.tensor(a.copy(), dtype=torch.float64, requires_grad=True) for a in twin.theta[:n_g]]
    opt_g = torch.optim.Adam(g_t, lr=float(twin.h[0]), betas=(spec.beta1, spec.beta2), eps=spec.eps)
    for s in range(2):
        ld, lg = gan.step(spec, m, 0, s, train_x)
        for k in range(K):
            rows = [int((int(philox.philox4x32_10([s, 0, philox.DOMAIN_BATCH, k * B + r], [spec.seed, 0])[0]) * 50) >> 32) for r in range(B)]
            loss_d, gd = gan.critic_loss_and_grads(spec, twin, train_x[rows], gan.latents(spec.seed, s, 0, 3 + k, B, 3), gan.gp_eps(spec.seed, s, 0, k, B))
            for p, g in zip(d_t, [a for gr in gd for a in gr]):
                p.grad = torch.tensor(g)
            opt_d.step()
            twin.theta[n_g:] = [p.detach().numpy().copy() for p in d_t]
        loss_g, gg = gan.wgan_generator_loss_and_grads(spec, twin, gan.latents(spec.seed, s, 0, 1, B, 3))
        for p, g in zip(g_t, [a for gr in gg for a in gr]):
            p.grad = torch.tensor(g)
        opt_g.step()
        twin.theta[:n_g] = [p.detach().numpy().copy() for p in g_t]
        assert abs(ld - loss_d) < 1e-9 and abs(lg - loss_g) < 1e-9
    assert m.t == 2
    for a, b in zip(m.theta, twin.theta):
        assert np.allclose(a, b, rtol=1e-9, atol=1e-12)


def test_wgan_gp_bf16_model_is_a_small_perturbation():
    spec, spec16 = _wspec(), _wspec(bf16=True)
    rng = np.random.default_rng(5)
    m = _member(spec, rng)
    real, z, eps = rng.standard_normal((4, 5)), rng.standard_normal((4, 3)), rng.random(4)
    la, ga = gan.critic_loss_and_grads(spec, m, real, z, eps)
    lb, gb = gan.critic_loss_and_grads(spec16, m, real, z, eps)
    assert 0 < abs(la - lb) < 5e-2 * max(1.0, abs(la))
    for (wa, _), (wb, _) in zip(ga, gb):
        assert np.linalg.norm(wa - wb) < 0.1 * np.linalg.norm(wa)
