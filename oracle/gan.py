"""`step` and `eval` for the GAN workload (oracle side).

The paper's GAN experiment (Section 4.3.1) trains a generator G and a
discriminator D with Adam, gives each member its own generator and
discriminator learning rate, copies both networks on exploit and scores members
with a sample-quality metric that is not the training loss.  This synthetic
stand-in keeps that structure with MLPs:

  step   one discriminator update on a mini-batch of B real rows and B generated
         rows (the generator is held fixed), then one generator update on B
         freshly generated rows through the UPDATED discriminator.  Losses are
         the logistic GAN losses, the generator's in its non-saturating form:
             L_D = mean softplus(-D(x)) + mean softplus(D(G(z)))
             L_G = mean softplus(-D(G(z')))
         With objective = "wgan_gp" the step is the paper's own (Section 4.3.1): K = n_critic
         updates of the discriminator ("critic"), then one update of the generator, on the
         WGAN-GP objective of Gulrajani et al. (2017),
             L_D = mean D(G(z)) - mean D(x) + gp_weight * mean (|grad_xhat D(xhat)|_2 - 1)^2,
             xhat = eps x + (1 - eps) G(z),  eps ~ U(0, 1) per row,
             L_G = -mean D(G(z')),
         with a fresh mini-batch, fresh latents and fresh eps for every critic update.  The
         paper gives neither the penalty weight nor the form of the interpolation; the reading
         is the cited paper's: gp_weight = 10, one eps per row.
  eval   minus the squared maximum mean discrepancy, with an RBF kernel
         k(a, b) = exp(-|a - b|^2 / (2 d)), d = data dimension, between n
         generated and n held-out real rows; biased (V-statistic) estimator
             MMD^2 = mean k(x, x') + mean k(y, y') - 2 mean k(x, y)
         with the diagonals included.

Latents z ~ N(0, I) come from Philox counter (step, member, DOMAIN_LATENT + s,
e // 4) for element e of the [B][d_z] array, s = 0 for the discriminator
update, 1 for the generator update, 2 for eval (step index 0); words (0, 1) and
(2, 3) of a counter each give one Box-Muller pair, so element e uses pair
(e % 4) // 2, cosine branch for even e, sine branch for odd e.
Adam's update count t advances once per step and is shared by both updates.
WGAN-GP: critic update k of a step draws its rows from batch counters k * B + r, its latents from
sub-stream 3 + k, and eps_r = (x + 0.5) / 2^32 from word 0 of counter (step, member, DOMAIN_GP_EPS,
k * B + r); the generator update uses sub-stream 1 as before.  The critic has had K (t - 1) + k + 1
updates when it takes update k of step t, and that is the count its bias correction uses; the
generator's count is t.
"""
import numpy as np

from . import nets, optim, philox, pbt

ROLE_LR_G, ROLE_LR_D = 3, 4
DOMAIN_GP_EPS = 14


class GanSpec:
    def __init__(self, g_dims, d_dims, batch, seed, roles=(ROLE_LR_G, ROLE_LR_D), g_hidden=nets.ACT_RELU,
                 g_out=nets.ACT_TANH, d_hidden=nets.ACT_LEAKY_RELU, beta1=0.5, beta2=0.999, eps=1e-8,
                 bf16_storage=False, objective="logistic", n_critic=1, gp_weight=10.0):
        self.g_dims, self.d_dims = list(g_dims), list(d_dims)
        assert self.g_dims[-1] == self.d_dims[0] and self.d_dims[-1] == 1
        self.batch, self.seed, self.roles = batch, seed, list(roles)
        self.g_hidden, self.g_out, self.d_hidden = g_hidden, g_out, d_hidden
        self.beta1, self.beta2, self.eps = beta1, beta2, eps
        self.q = nets.round_bf16 if bf16_storage else nets.identity
        self.n_g = len(self.g_dims) - 1            # generator layers come first in theta
        assert objective in ("logistic", "wgan_gp")
        self.objective, self.n_critic, self.gp_weight = objective, int(n_critic), float(gp_weight)


def latents(seed, c0, member, substream, n_rows, d_z):
    e = np.arange(n_rows * d_z)
    w = philox.words(seed, c0, member, philox.DOMAIN_LATENT + substream, e // 4)
    pair = (e % 4) // 2
    n_cos, n_sin = philox.normal_pairs(w[e, 2 * pair], w[e, 2 * pair + 1])
    return np.where(e % 2 == 0, n_cos, n_sin).reshape(n_rows, d_z)


def new_member(spec, g_layers, d_layers, h, index):
    flat = [np.array(a, dtype=np.float64) for Wb in list(g_layers) + list(d_layers) for a in Wb]
    opt = {"s0": [np.zeros_like(a) for a in flat], "s1": [np.zeros_like(a) for a in flat]}
    return pbt.Member(flat, h, opt, index)


def g_params(spec, m):
    return [(m.theta[2 * l], m.theta[2 * l + 1]) for l in range(spec.n_g)]


def d_params(spec, m):
    L = len(m.theta) // 2
    return [(m.theta[2 * l], m.theta[2 * l + 1]) for l in range(spec.n_g, L)]


def _adam_range(spec, m, first_layer, grads, lr, t=None):
    t = m.t if t is None else t
    for k, g in enumerate([a for gr in grads for a in gr]):
        j = 2 * first_layer + k
        m.theta[j], m.opt["s0"][j], m.opt["s1"][j] = optim.adam(
            m.theta[j], g, m.opt["s0"][j], m.opt["s1"][j], t, lr, spec.beta1, spec.beta2, spec.eps, 0.0)


def generate(spec, m, z):
    return nets.mlp_forward(g_params(spec, m), z, spec.g_hidden, spec.g_out, q=spec.q)


def d_loss_and_grads(spec, m, real, z):
    fake, _ = generate(spec, m, z)
    x = np.concatenate([real, fake], axis=0)
    t = np.concatenate([np.ones(len(real)), np.zeros(len(fake))])
    logits, cache = nets.mlp_forward(d_params(spec, m), x, spec.d_hidden, q=spec.q)
    # mean over the real rows plus mean over the generated rows
    l_real, d_real = nets.logistic_loss(logits[:len(real)], t[:len(real)])
    l_fake, d_fake = nets.logistic_loss(logits[len(real):], t[len(real):])
    grads, _ = nets.mlp_backward(d_params(spec, m), cache, np.concatenate([d_real, d_fake], axis=0), spec.d_hidden, q=spec.q)
    return l_real + l_fake, grads


def g_loss_and_grads(spec, m, z):
    fake, g_cache = generate(spec, m, z)
    logits, d_cache = nets.mlp_forward(d_params(spec, m), fake, spec.d_hidden, q=spec.q)
    loss, dlogits = nets.logistic_loss(logits, np.ones(len(fake)))
    _, d_fake = nets.mlp_backward(d_params(spec, m), d_cache, dlogits, spec.d_hidden, q=spec.q)
    grads, _ = nets.mlp_backward(g_params(spec, m), g_cache, d_fake, spec.g_hidden, spec.g_out, q=spec.q)
    return loss, grads


def critic_input_gradient(spec, d_layers, x):
    """D(x) and its gradient with respect to x, row by row: the backward pass of the critic started from
    d out = 1.  Returns (out, g [n][d], the per-layer pre-activation gradients dz, the forward cache)."""
    q = spec.q
    out, (ins, zs) = nets.mlp_forward(d_layers, x, spec.d_hidden, q=q)
    L = len(d_layers)
    dz = [None] * L
    da = np.ones((len(x), 1))
    for l in range(L - 1, -1, -1):
        dz[l] = q(da * nets.act_grad(zs[l], spec.d_hidden if l < L - 1 else nets.ACT_NONE))
        da = dz[l] @ q(d_layers[l][0]).T
    return out, da, dz, (ins, zs)


def gradient_penalty_and_grads(spec, d_layers, xhat):
    """gp_weight * mean_r (|g_r| - 1)^2 with g_r = grad_x D(xhat_r), and its gradient with respect to the
    critic's weights.  g = dz_0 W_0^T with dz_l = (dz_{l+1} W_{l+1}^T) * act'(z_l): it is linear in every
    W_l, and the activation slopes are piecewise constant, so the gradient of the penalty flows through
    that chain in the opposite direction: with c = d penalty / d g,
        d penalty / d W_0 = c^T dz_0,  c_1 = (c W_0) * act'(z_0),  d penalty / d W_1 = c_1^T dz_1,  ...
    The biases do not enter g."""
    q = spec.q
    n = len(xhat)
    _, g, dz, (_, zs) = critic_input_gradient(spec, d_layers, xhat)
    norm = np.sqrt((g * g).sum(axis=1))
    penalty = spec.gp_weight * np.mean((norm - 1.0) ** 2)
    c = q((2.0 * spec.gp_weight / n) * ((norm - 1.0) / norm)[:, None] * g)
    grads = []
    for l, (W, b) in enumerate(d_layers):
        grads.append((c.T @ dz[l], np.zeros_like(b)))
        if l < len(d_layers) - 1:
            c = q((c @ q(W)) * nets.act_grad(zs[l], spec.d_hidden))
    return penalty, grads


def critic_loss_and_grads(spec, m, real, z, eps):
    """WGAN-GP critic loss on one mini-batch (the generator is held fixed) and its gradient."""
    q = spec.q
    fake, _ = generate(spec, m, z)
    xr, xf = q(np.asarray(real, dtype=np.float64)), q(fake)          # what the data fetch and the generator hand on
    D = d_params(spec, m)
    logits, cache = nets.mlp_forward(D, np.concatenate([xr, xf], axis=0), spec.d_hidden, q=q)
    B = len(real)
    wasserstein = logits[B:].mean() - logits[:B].mean()
    d_out = np.concatenate([np.full((B, 1), -1.0 / B), np.full((len(fake), 1), 1.0 / len(fake))], axis=0)
    grads_w, _ = nets.mlp_backward(D, cache, d_out, spec.d_hidden, q=q)
    e = np.asarray(eps, dtype=np.float64)[:, None]
    penalty, grads_p = gradient_penalty_and_grads(spec, D, e * xr + (1.0 - e) * xf)
    return wasserstein + penalty, [(gw + pw, gb + pb) for (gw, gb), (pw, pb) in zip(grads_w, grads_p)]


def wgan_generator_loss_and_grads(spec, m, z):
    fake, g_cache = generate(spec, m, z)
    logits, d_cache = nets.mlp_forward(d_params(spec, m), fake, spec.d_hidden, q=spec.q)
    loss = -logits.mean()
    _, d_fake = nets.mlp_backward(d_params(spec, m), d_cache, np.full(logits.shape, -1.0 / len(fake)), spec.d_hidden, q=spec.q)
    grads, _ = nets.mlp_backward(g_params(spec, m), g_cache, d_fake, spec.g_hidden, spec.g_out, q=spec.q)
    return loss, grads


def gp_eps(seed, s, member, k, batch):
    x = philox.words(seed, s, member, DOMAIN_GP_EPS, k * batch + np.arange(batch))[..., 0]
    return philox.unit_open(x)


def step_wgan_gp(spec, m, i, s, train_x):
    """One `step` of the paper's GAN experiment: n_critic critic updates, then one generator update.
    Returns (L_D of the last critic update, L_G), each before its own update."""
    B, K, dz = spec.batch, spec.n_critic, spec.g_dims[0]
    m.t += 1
    lr_g = m.h[spec.roles.index(ROLE_LR_G)]
    lr_d = m.h[spec.roles.index(ROLE_LR_D)]
    for k in range(K):
        rows = philox.bounded(philox.words(spec.seed, s, i, philox.DOMAIN_BATCH, k * B + np.arange(B))[..., 0], len(train_x))
        loss_d, gd = critic_loss_and_grads(spec, m, train_x[rows], latents(spec.seed, s, i, 3 + k, B, dz), gp_eps(spec.seed, s, i, k, B))
        _adam_range(spec, m, spec.n_g, gd, lr_d, t=K * (m.t - 1) + k + 1)
    loss_g, gg = wgan_generator_loss_and_grads(spec, m, latents(spec.seed, s, i, 1, B, dz))
    _adam_range(spec, m, 0, gg, lr_g)
    return loss_d, loss_g


def step(spec, m, i, s, train_x):
    """One `step`.  Returns (L_D, L_G), each before its own update."""
    if spec.objective == "wgan_gp":
        return step_wgan_gp(spec, m, i, s, train_x)
    rows = philox.bounded(philox.words(spec.seed, s, i, philox.DOMAIN_BATCH, np.arange(spec.batch))[..., 0], len(train_x))
    m.t += 1
    lr_g = m.h[spec.roles.index(ROLE_LR_G)]
    lr_d = m.h[spec.roles.index(ROLE_LR_D)]
    loss_d, gd = d_loss_and_grads(spec, m, train_x[rows], latents(spec.seed, s, i, 0, spec.batch, spec.g_dims[0]))
    _adam_range(spec, m, spec.n_g, gd, lr_d)
    loss_g, gg = g_loss_and_grads(spec, m, latents(spec.seed, s, i, 1, spec.batch, spec.g_dims[0]))
    _adam_range(spec, m, 0, gg, lr_g)
    return loss_d, loss_g


def rbf_mmd2(x, y):
    """Biased squared MMD with k(a, b) = exp(-|a - b|^2 / (2 d))."""
    d = x.shape[1]

    def kmean(a, b):
        sq = (a * a).sum(1)[:, None] + (b * b).sum(1)[None, :] - 2.0 * (a @ b.T)
        return np.exp(-sq / (2.0 * d)).mean()
    return kmean(x, x) + kmean(y, y) - 2.0 * kmean(x, y)


def evaluate(spec, m, i, eval_x):
    """`eval`: minus MMD^2 between len(eval_x) generated rows and the held-out rows."""
    z = latents(spec.seed, 0, i, 2, len(eval_x), spec.g_dims[0])
    fake, _ = generate(spec, m, z)
    return -rbf_mmd2(spec.q(fake), spec.q(np.asarray(eval_x, dtype=np.float64)))
