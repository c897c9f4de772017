"""Pins on WHERE the oracle rounds to bfloat16 under "bf16 compute with fp32 master weights".

The rounding model is part of the written specification of the bf16 workloads (operands of every
dense contraction and every tensor kept between two operations are bf16 values; biases, logits,
statistics, losses and the optimiser are not).  These tests fail when a rounding point of the
oracle is dropped, added or moved:

  * hand-computed scalar networks whose values sit on bfloat16 midpoints, so that every rounding
    point changes a number that is checked against a literal;
  * for every workload, the ordered list of tensors that pass through the rounding hook during one
    loss-and-gradient evaluation, and a check that switching any single one of them off changes
    the result.
"""
import math

import numpy as np

from oracle import a2c, gan, nets, transformer as tf

R = nets.round_bf16


def _a(v):
    return np.array([[v]], dtype=np.float64)


# ---- bfloat16 itself ---------------------------------------------------------------------------

def test_round_bf16_ties_go_to_even_mantissas():
    # 8 significant bits: spacing 1/128 in [1, 2), 1/256 in [0.5, 1), 1/512 in [0.25, 0.5)
    cases = {1 + 1 / 256: 1.0, 1 + 3 / 256: 1 + 4 / 256, 1.5 + 1 / 256: 1.5, 199.5 / 256: 200 / 256,
             1297 / 1024: 1296 / 1024, 133 / 256 + 1 / 1024: 133 / 256, -(1 + 3 / 256): -(1 + 4 / 256)}
    for x, want in cases.items():
        assert float(R(np.array([x]))[0]) == want, x


# ---- hand-computed two-layer networks ----------------------------------------------------------
# Network: out = a1 * W2 + b2, a1 = act(x * W1 + b1), all 1 x 1.  Every literal below was worked out
# by hand from the rounding rule above; none comes from the oracle.

X, W1, B1, W2, B2, DOUT = 1 + 1 / 256, 1 + 3 / 256, 257 / 1024, 133 / 256 + 1 / 1024, 0.0, 1.5 + 1 / 256


def _relu_case(q=R):
    params = [(_a(W1), np.array([B1])), (_a(W2), np.array([B2]))]
    out, cache = nets.mlp_forward(params, _a(X), nets.ACT_RELU, q=q)
    grads, dx = nets.mlp_backward(params, cache, _a(DOUT), nets.ACT_RELU, q=q)
    return out, cache, grads, dx


def test_mlp_rounding_points_relu_hand_case():
    """x = 1 + 1/256 -> 1 (tie to even).  W1 = 1 + 3/256 -> 1 + 4/256 = 1040/1024.
    z1 = 1 * 1040/1024 + 257/1024 = 1297/1024 (the bias 257/1024 is NOT rounded: as bf16 it would be 1/4).
    a1 = bf16(relu(z1)) = 1296/1024 (1297/8 = 162.125 -> 162).  W2 = 133/256 + 1/1024 -> 133/256.
    out = 1296/1024 * 133/256 = 172368/262144, kept unrounded (bf16 would give 168/256).
    Backward from d_out = 1.5 + 1/256 -> dz2 = 1.5 (tie to even):
    dW2 = a1 * dz2 = 1.8984375, db2 = 1.5; da1 = dz2 * bf16(W2) = 199.5/256 -> dz1 = 200/256 (tie to even);
    dW1 = bf16(x) * dz1 = 0.78125, db1 = 0.78125; dx = dz1 * bf16(W1) = 0.78125 * 1.015625."""
    out, cache, grads, dx = _relu_case()
    assert out[0, 0] == 172368 / 262144
    assert cache[0][0][0, 0] == 1.0 and cache[0][1][0, 0] == 1296 / 1024      # stored layer inputs
    assert cache[1][0][0, 0] == 1296 / 1024                                   # stored hidden pre-activation
    assert grads[1][0][0, 0] == 1.8984375 and grads[1][1][0] == 1.5
    assert grads[0][0][0, 0] == 0.78125 and grads[0][1][0] == 0.78125
    assert dx[0, 0] == 0.78125 * 1.015625


def test_mlp_without_rounding_gives_the_exact_products():
    out, _, grads, dx = _relu_case(q=nets.identity)
    z1 = X * W1 + B1
    assert out[0, 0] == z1 * W2 and grads[1][0][0, 0] == z1 * DOUT
    assert grads[0][0][0, 0] == X * (DOUT * W2) and dx[0, 0] == W1 * (DOUT * W2)


def test_mlp_rounding_points_tanh_hand_case():
    """The hidden activation acts on the UNROUNDED pre-activation; its derivative in the backward pass is
    taken at the ROUNDED, stored one.  z1 = 1 * 1 + 3/256 = 1.01171875, stored as bf16 1.015625.
    tanh(1.01171875) = 0.76647 -> a1 = 196/256 (tanh of the stored 1.015625 = 0.76901 would give 197/256).
    1 - tanh(1.015625)^2 = 0.410055 -> dz1 = 210/512 (at the unrounded z1: 0.412521 -> 211/512)."""
    params = [(_a(1.0), np.array([3 / 256])), (_a(1.0), np.array([0.0]))]
    out, cache = nets.mlp_forward(params, _a(1.0), nets.ACT_TANH, q=R)
    assert 195.5 / 256 < math.tanh(1.01171875) < 196.5 / 256 < math.tanh(1.015625) < 197.5 / 256
    assert out[0, 0] == 196 / 256 and cache[1][0][0, 0] == 1.015625
    grads, _ = nets.mlp_backward(params, cache, _a(1.0), nets.ACT_TANH, q=R)
    assert 209.5 / 512 < 1 - math.tanh(1.015625) ** 2 < 210.5 / 512 < 1 - math.tanh(1.01171875) ** 2 < 211.5 / 512
    assert grads[0][0][0, 0] == 210 / 512 and grads[0][1][0] == 210 / 512


def test_output_nonlinearity_keeps_its_pre_activation_rounded_and_its_value_not():
    """A generator's tanh output: the last pre-activation is stored (rounded) for the backward pass,
    the output itself leaves unrounded (the discriminator rounds it as its own input)."""
    params = [(_a(1.0), np.array([3 / 256]))]
    out, cache = nets.mlp_forward(params, _a(1.0), nets.ACT_RELU, out_act=nets.ACT_TANH, q=R)
    assert out[0, 0] == math.tanh(1.01171875) and cache[1][0][0, 0] == 1.015625
    grads, _ = nets.mlp_backward(params, cache, _a(1.0), nets.ACT_RELU, out_act=nets.ACT_TANH, q=R)
    assert grads[0][1][0] == 210 / 512


# ---- which tensors are rounded, in order, for every workload -----------------------------------

class _Recorder:
    """Rounding hook that lists what it is given and can leave one call (by position) unrounded."""

    def __init__(self, skip=None):
        self.shapes, self.skip = [], skip

    def __call__(self, x):
        k = len(self.shapes)
        self.shapes.append(tuple(np.shape(x)))
        return np.asarray(x, dtype=np.float64) if k == self.skip else R(x)


def _every_point_is_live(run, n_points, sign_only=()):
    """run(q) -> flat result vector; leaving any single rounding point out must change it, except the
    points listed in sign_only: stored ReLU / LeakyReLU pre-activations, of which the backward pass uses
    the sign alone, which rounding keeps."""
    base = run(_Recorder())
    for k in range(n_points):
        r = run(_Recorder(skip=k))
        assert r.shape == base.shape
        assert np.array_equal(r, base) == (k in sign_only), "rounding point %d: effect %s" % (k, not np.array_equal(r, base))
    return base


def test_mlp_rounding_points_in_order():
    dims, B = [5, 7, 6, 3], 4
    rng = np.random.default_rng(1)
    params = [(rng.standard_normal((a, b)), rng.standard_normal(b)) for a, b in zip(dims[:-1], dims[1:])]
    x, labels = rng.standard_normal((B, dims[0])), rng.integers(0, 3, B)
    rec = _Recorder()
    nets.classifier_loss_and_grads(params, x, labels, nets.ACT_GELU, q=rec)
    want = [(B, 5),                                   # mini-batch
            (5, 7), (B, 7), (B, 7),                   # layer 0: weights, stored pre-activation, activation
            (7, 6), (B, 6), (B, 6),                   # layer 1
            (6, 3),                                   # output layer: weights only (logits stay unrounded)
            (B, 3), (6, 3),                           # backward: logit gradient, weights for the input gradient
            (B, 6), (7, 6), (B, 7), (5, 7)]           # hidden gradients and the weights they pass through
    assert rec.shapes == want

    def run(q):
        loss, grads = nets.classifier_loss_and_grads(params, x, labels, nets.ACT_GELU, q=q)
        return np.concatenate([[loss]] + [a.ravel() for g in grads for a in g])
    # (the last point, bf16(W_0) for the gradient with respect to the network input, feeds nothing here)
    _every_point_is_live(run, len(want) - 1)


def test_transformer_rounding_points_in_order():
    V, d, H, f, L, S, B = 11, 6, 2, 10, 1, 4, 3
    n, dh = B * S, d // H
    spec = tf.TransformerSpec(V, d, H, f, L, S, B, seed=3, bf16_storage=True)
    rng = np.random.default_rng(0)
    arrs = [rng.standard_normal(s) * 0.3 for _, s in spec.param_shapes()]
    m = tf.new_member(spec, arrs, np.array([1e-3, 0.2, 0.1], dtype=np.float32), 0)
    seqs = rng.integers(0, V, (B, S + 1))
    rec = _Recorder()
    spec.q = rec
    tf.loss_and_grads(spec, m, seqs, 0, 0)
    attn, heads = (B, H, S, S), (B, H, S, dh)
    want = [(V, d), (S, d), (B, S, d),                # token table, position table, their sum
            (n, d), (d, 3 * d), (n, 3 * d),           # LN1 output, Wqkv, QKV
            attn, attn, attn, heads,                  # raw scores, probabilities, dropped probabilities, P V
            (d, d), (n, d), (n, d),                   # Wo, attention output, residual sum
            (n, d), (d, f), (n, f), (n, f), (n, f),   # LN2 output, W1, pre-activation, ReLU, dropped ReLU
            (f, d), (n, d), (n, d),                   # W2, feed-forward output, residual sum
            (n, d), (d, V),                           # final LN output, head weights (logits stay unrounded)
            (n, V), (d, V), (n, d), (n, d),           # backward: logit gradient, head weights, d(final LN out), d(residual)
            (n, d), (f, d), (n, f), (n, f),           # feed-forward: masked d(out), W2, d(dropped hidden), d(pre-activation)
            (d, f), (n, d), (n, d),                   # W1, d(LN2 out), residual gradient
            (n, d), (d, d), (n, d),                   # attention: masked d(out), Wo, d(merged heads)
            heads, attn, attn, heads, heads,          # dV, d(dropped probabilities), d(scores), dQ, dK
            (d, 3 * d), (n, d), (n, d)]               # Wqkv, d(LN1 out), residual gradient
    assert rec.shapes == want

    def run(q):
        spec.q = q
        loss, grads = tf.loss_and_grads(spec, m, seqs, 0, 0)
        return np.concatenate([[loss]] + [g.ravel() for g in grads])
    _every_point_is_live(run, len(want), sign_only=[want.index((n, f))])


def test_gan_rounding_points_in_order():
    B, zd = 4, 3
    spec = gan.GanSpec([zd, 5, 6], [6, 7, 1], B, seed=1, bf16_storage=True)
    rng = np.random.default_rng(2)
    g = [(rng.standard_normal((a, b)), rng.standard_normal(b)) for a, b in ((zd, 5), (5, 6))]
    dn = [(rng.standard_normal((a, b)), rng.standard_normal(b)) for a, b in ((6, 7), (7, 1))]
    m = gan.new_member(spec, g, dn, np.array([1e-3, 1e-3], dtype=np.float32), 0)
    real, z = rng.standard_normal((B, 6)), rng.standard_normal((B, zd))
    rec = _Recorder()
    spec.q = rec
    gan.d_loss_and_grads(spec, m, real, z)
    gen_fwd = [(B, zd), (zd, 5), (B, 5), (B, 5), (5, 6), (B, 6)]      # latents; hidden layer; output weights, stored tanh pre-activation
    want_d = gen_fwd + [(2 * B, 6), (6, 7), (2 * B, 7), (2 * B, 7), (7, 1),         # discriminator on real + generated rows
                        (2 * B, 1), (7, 1), (2 * B, 7), (6, 7)]                     # its backward pass
    assert rec.shapes == want_d
    rec = _Recorder()
    spec.q = rec
    gan.g_loss_and_grads(spec, m, z)
    want_g = gen_fwd + [(B, 6), (6, 7), (B, 7), (B, 7), (7, 1), (B, 1), (7, 1), (B, 7), (6, 7),
                        (B, 6), (5, 6), (B, 5), (zd, 5)]                            # back through the tanh output and the generator
    assert rec.shapes == want_g
    rec = _Recorder()
    spec.q = rec
    gan.evaluate(spec, m, 0, rng.standard_normal((8, 6)))
    assert rec.shapes == [(8, zd), (zd, 5), (8, 5), (8, 5), (5, 6), (8, 6), (8, 6), (8, 6)]   # ..., generated rows, held-out rows

    def run(q):
        spec.q = q
        loss, grads = gan.g_loss_and_grads(spec, m, z)
        return np.concatenate([[loss]] + [a.ravel() for gr in grads for a in gr])
    _every_point_is_live(run, len(want_g) - 1, sign_only=[2, 8])      # ReLU and LeakyReLU pre-activations


def test_actor_critic_rounding_points_in_order():
    B, T, na = 3, 2, 4
    spec = a2c.A2CSpec([6, 5], na, B, T, seed=1, bf16_storage=True)
    rng = np.random.default_rng(3)
    layers = [(rng.standard_normal((a, b)), rng.standard_normal(b)) for a, b in ((6, 5), (5, na + 1))]
    m = a2c.new_member(spec, layers, np.array([1e-3, 1e-2], dtype=np.float32), 0)
    obs = rng.standard_normal((B, T + 1, 6))
    actions, rewards = rng.integers(0, na, (B, T)), rng.standard_normal((B, T))
    rec = _Recorder()
    spec.q = rec
    a2c.loss_and_grads(spec, m, obs, actions, rewards)
    rows = B * (T + 1)
    want = [(rows, 6), (6, 5), (rows, 5), (rows, 5), (5, na + 1),       # observations, torso layer, head weights (head outputs unrounded)
            (rows, na + 1), (5, na + 1), (rows, 5), (6, 5)]             # gradient of the head outputs, and back through the torso
    assert rec.shapes == want

    def run(q):
        spec.q = q
        loss, grads = a2c.loss_and_grads(spec, m, obs, actions, rewards)
        return np.concatenate([[loss]] + [a.ravel() for gr in grads for a in gr])
    _every_point_is_live(run, len(want) - 1, sign_only=[2])


def test_wgan_gp_rounding_points_in_order():
    B, zd = 4, 3
    spec = gan.GanSpec([zd, 5, 6], [6, 7, 1], B, seed=1, bf16_storage=True, objective="wgan_gp", n_critic=2)
    rng = np.random.default_rng(2)
    g = [(rng.standard_normal((a, b)), rng.standard_normal(b)) for a, b in ((zd, 5), (5, 6))]
    dn = [(rng.standard_normal((a, b)), rng.standard_normal(b)) for a, b in ((6, 7), (7, 1))]
    m = gan.new_member(spec, g, dn, np.array([1e-3, 1e-3], dtype=np.float32), 0)
    real, z, eps = rng.standard_normal((B, 6)), rng.standard_normal((B, zd)), rng.random(B)
    rec = _Recorder()
    spec.q = rec
    gan.critic_loss_and_grads(spec, m, real, z, eps)
    want = [(B, zd), (zd, 5), (B, 5), (B, 5), (5, 6), (B, 6),                   # generator forward
            (B, 6), (B, 6),                                                      # real rows and generated rows as handed on
            (2 * B, 6), (6, 7), (2 * B, 7), (2 * B, 7), (7, 1),                  # critic on real + generated rows
            (2 * B, 1), (7, 1), (2 * B, 7), (6, 7),                              # its backward pass (Wasserstein terms)
            (B, 6), (6, 7), (B, 7), (B, 7), (7, 1),                              # critic on the interpolated rows
            (B, 1), (7, 1), (B, 7), (6, 7),                                      # input-gradient pass from d out = 1
            (B, 6), (6, 7), (B, 7)]                                              # d penalty / d g, and its way back through W_0
    assert rec.shapes == want

    def run(q):
        spec.q = q
        loss, grads = gan.critic_loss_and_grads(spec, m, real, z, eps)
        return np.concatenate([[loss]] + [a.ravel() for gr in grads for a in gr])
    # The critic's forward pass on the interpolated rows (17-21) enters the penalty only through the LeakyReLU
    # slopes, i.e. through signs; 2, 10 are ReLU / LeakyReLU pre-activations, 5 is kept for the generator's own
    # backward pass, 6-8 round values that are rounded again (or are already bf16), 13 and 22 are +-1/B and 1,
    # 16 feeds the unused gradient with respect to the critic's input.  Every other point must change the result.
    base = run(_Recorder())
    live = [k for k in range(len(want)) if not np.array_equal(run(_Recorder(skip=k)), base)]
    assert set(live) >= {0, 1, 3, 4, 9, 11, 12, 14, 15, 23, 24, 25, 26, 27, 28}, live
