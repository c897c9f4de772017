"""Pins for the oracle's actor-critic workload: return scan against its double-loop definition,
entropy closed form, finite differences of the surrogate loss, history semantics."""
import math
import numpy as np

from oracle import a2c, nets


def _member(spec, rng, h=(1e-3, 1e-2)):
    d = spec.dims
    layers = [(rng.standard_normal((a, b)) * 0.5, rng.standard_normal(b) * 0.1) for a, b in zip(d[:-1], d[1:])]
    return a2c.new_member(spec, layers, h, 0)


def test_returns_against_double_loop():
    rng = np.random.default_rng(0)
    r, boot, g = rng.standard_normal((3, 6)), rng.standard_normal(3), 0.9
    R = a2c.returns(r, boot, g)
    for b in range(3):
        for t in range(6):
            ref = sum(g ** (k - t) * r[b, k] for k in range(t, 6)) + g ** (6 - t) * boot[b]
            assert abs(R[b, t] - ref) < 1e-13
    assert np.allclose(a2c.returns(np.ones((1, 4)), [0.0], 1.0), [[4, 3, 2, 1]])


def test_entropy_and_logprob_closed_forms():
    lp, ent = a2c.policy_terms(np.zeros((2, 18)))
    assert np.allclose(ent, math.log(18)) and np.allclose(lp, -math.log(18))      # uniform policy
    lp, ent = a2c.policy_terms(np.array([[50.0, 0.0, 0.0]]))
    assert ent[0] < 1e-19 and abs(lp[0, 0]) < 1e-20                               # deterministic policy
    p = np.array([0.2, 0.5, 0.3])
    lp, ent = a2c.policy_terms(np.log(p)[None])
    assert abs(ent[0] + (p * np.log(p)).sum()) < 1e-15


def test_surrogate_gradients_fd():
    spec = a2c.A2CSpec([5, 7, 6], n_actions=4, batch=3, unroll=5, seed=1)
    rng = np.random.default_rng(2)
    m = _member(spec, rng)
    obs = rng.standard_normal((3, 6, 5))
    act = rng.integers(0, 4, (3, 5))
    rew = rng.standard_normal((3, 5))
    loss, grads = a2c.loss_and_grads(spec, m, obs, act, rew)
    # returns and advantages are constants of the surrogate: freeze them at the base point
    out = nets.mlp_forward(a2c.params_of(m), obs.reshape(18, 5), spec.hidden_act)[0].reshape(3, 6, 5)
    R = a2c.returns(rew, out[:, 5, 4], spec.gamma)
    adv = R - out[:, :5, 4]
    ec = float(m.h[1])

    def surrogate():
        o = nets.mlp_forward(a2c.params_of(m), obs.reshape(18, 5), spec.hidden_act)[0].reshape(3, 6, 5)
        lp, ent = a2c.policy_terms(o[:, :5, :4])
        lpa = np.take_along_axis(lp, act[..., None], -1)[..., 0]
        return (-(adv * lpa).sum() + 0.5 * ((R - o[:, :5, 4]) ** 2).sum() - ec * ent.sum()) / 15

    assert abs(surrogate() - loss) < 1e-13
    flat_g = [a for gr in grads for a in gr]
    e = 1e-6
    for arr, g in zip(m.theta, flat_g):
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = arr[idx]
            arr[idx] = old + e
            lp_ = surrogate()
            arr[idx] = old - e
            lm_ = surrogate()
            arr[idx] = old
            assert abs((lp_ - lm_) / (2 * e) - g[idx]) <= 1e-6 * max(1.0, abs(g[idx]))


def test_step_history_and_eval():
    spec = a2c.A2CSpec([5, 7, 6], n_actions=4, batch=3, unroll=5, seed=1)
    rng = np.random.default_rng(3)
    m = _member(spec, rng)
    pool_obs, pool_act, pool_rew = rng.standard_normal((20, 6, 5)), rng.integers(0, 4, (20, 5)), rng.standard_normal((20, 5))
    assert a2c.evaluate(spec, m) == -np.inf
    rets = []
    for s in range(13):
        a2c.step(spec, m, 0, s, pool_obs, pool_act, pool_rew)
        from oracle import philox
        idx = [(int(philox.philox4x32_10([s, 0, philox.DOMAIN_BATCH, r], [1, 0])[0]) * 20) >> 32 for r in range(3)]
        rets.append(np.float32(pool_rew[idx].sum(axis=1).mean()))
        assert abs(float(a2c.evaluate(spec, m)) - float(np.mean(np.array(rets[-10:], dtype=np.float64)))) < 1e-6
    assert len(m.hist) == 10 and m.t == 13


def test_entropy_cost_pushes_towards_uniform():
    spec = a2c.A2CSpec([5, 7, 6], n_actions=4, batch=3, unroll=5, seed=1)
    rng = np.random.default_rng(4)
    obs, act, rew = rng.standard_normal((3, 6, 5)), rng.integers(0, 4, (3, 5)), np.zeros((3, 5))
    lo, hi = _member(spec, np.random.default_rng(5), h=(1e-3, 0.0)), _member(spec, np.random.default_rng(5), h=(1e-3, 1.0))
    l0, _ = a2c.loss_and_grads(spec, lo, obs, act, rew)
    l1, _ = a2c.loss_and_grads(spec, hi, obs, act, rew)
    out = nets.mlp_forward(a2c.params_of(lo), obs.reshape(18, 5), spec.hidden_act)[0].reshape(3, 6, 5)
    _, ent = a2c.policy_terms(out[:, :5, :4])
    assert abs((l0 - l1) - ent.mean()) < 1e-12
