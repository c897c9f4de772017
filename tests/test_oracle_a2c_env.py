"""Pins of the on-policy unroll generator of the actor-critic oracle (oracle/a2c_env.py)."""
import math

import numpy as np

from oracle import a2c, a2c_env as env_, nets, philox


def _env(nz=3, na=4, d=6, seed=0, **kw):
    rng = np.random.default_rng(seed)
    return env_.Environment(0.5 * rng.standard_normal((nz, nz)), rng.standard_normal((nz, na)), rng.standard_normal((d, nz)),
                            rng.standard_normal(nz), **kw)


def _spec(na=4, d=6, B=5, T=3, seed=7):
    return a2c.A2CSpec([d, 8], na, B, T, seed)


def _params(spec, rng, scale=0.3):
    return [(scale * rng.standard_normal((a, b)), scale * rng.standard_normal(b)) for a, b in zip(spec.dims[:-1], spec.dims[1:])]


def test_normal_stream_counter_assignment_and_moments():
    x = env_.normals(9, 4, 2, 1, 50001)
    assert abs(x.mean()) < 0.02 and abs(x.var() - 1.0) < 0.02 and abs((x ** 3).mean()) < 0.05
    # element e = word pair (e % 4) // 2 of counter e // 4; cosine branch for even e, sine for odd e
    for e in (0, 1, 2, 3, 4, 4101, 50000):
        w = philox.philox4x32_10([4, 2, env_.DOMAIN_ENV + 1, e // 4], [9, 0])
        k = 2 * ((e % 4) // 2)
        u1, u2 = (int(w[k]) + 0.5) / 2 ** 32, (int(w[k + 1]) + 0.5) / 2 ** 32
        r = math.sqrt(-2.0 * math.log(u1))
        want = r * (math.cos(2 * math.pi * u2) if e % 2 == 0 else math.sin(2 * math.pi * u2))
        assert abs(x[e] - want) < 1e-12
    u = env_.uniforms(9, 4, 2, 2, 7)
    for e in (0, 6):
        assert u[e] == (int(philox.philox4x32_10([4, 2, env_.DOMAIN_ENV + 2, e], [9, 0])[0]) + 0.5) / 2 ** 32
    # different streams and members do not repeat each other
    assert not np.array_equal(env_.normals(9, 4, 2, 0, 16), env_.normals(9, 4, 2, 1, 16))
    assert not np.array_equal(env_.normals(9, 4, 2, 0, 16), env_.normals(9, 4, 3, 0, 16))


def test_action_choice_is_the_inverse_cdf():
    logits = np.log(np.array([[0.2, 0.3, 0.5]]))
    for u, want in ((0.0001, 0), (0.1999, 0), (0.2001, 1), (0.4999, 1), (0.5001, 2), (0.9999, 2)):
        a, margin = env_.choose(logits, np.array([u]))
        assert a[0] == want
        assert abs(margin[0] - min(abs(u - 0.2), abs(u - 0.5))) < 1e-12
    # shift invariance of softmax, and frequencies over many uniform draws
    a1, _ = env_.choose(logits + 100.0, np.array([0.3]))
    assert a1[0] == 1
    u = env_.uniforms(3, 0, 0, 2, 40000)
    a, _ = env_.choose(np.repeat(logits, len(u), axis=0), u)
    freq = np.bincount(a, minlength=3) / len(u)
    assert np.all(np.abs(freq - [0.2, 0.3, 0.5]) < 0.01)


def test_rollout_follows_the_linear_system_step_by_step():
    """Without noise the latent follows z' = A z + B[:, a] exactly; checked against explicit loops."""
    e = _env(obs_noise=0.0, reward_noise=0.0, trans_noise=0.0)
    spec = _spec()
    params = _params(spec, np.random.default_rng(1))
    obs, actions, rewards, _ = env_.rollout(spec, e, params, member=2, step=5)
    z0 = env_.normals(spec.seed, 5, 2, 0, spec.batch * e.n_z).reshape(spec.batch, e.n_z)
    for r in range(spec.batch):
        z = z0[r].copy()
        for t in range(spec.unroll + 1):
            assert np.allclose(obs[r, t], e.C @ z, rtol=1e-6, atol=1e-6)
            if t < spec.unroll:
                assert abs(rewards[r, t] - float(e.w @ z)) < 1e-5
                z = e.A @ z + e.B[:, actions[r, t]]
    assert obs.dtype == np.float32 and rewards.dtype == np.float32


def test_noise_enters_with_its_scale_and_its_own_stream():
    spec = _spec(B=4, T=2)
    params = _params(spec, np.random.default_rng(2))
    quiet = _env(obs_noise=0.0, reward_noise=0.0, trans_noise=0.0)
    o0, a0, r0, _ = env_.rollout(spec, quiet, params, 0, 0)
    noisy_obs = _env(obs_noise=0.5, reward_noise=0.0, trans_noise=0.0)
    o1, a1, r1, _ = env_.rollout(spec, noisy_obs, params, 0, 0, forced_actions=a0)
    xi = env_.normals(spec.seed, 0, 0, 1, 4 * 3 * 6).reshape(4, 3, 6)
    assert np.allclose(o1 - o0, 0.5 * xi, atol=1e-6) and np.allclose(r1, r0, atol=1e-6)
    noisy_rew = _env(obs_noise=0.0, reward_noise=0.25, trans_noise=0.0)
    _, _, r2, _ = env_.rollout(spec, noisy_rew, params, 0, 0, forced_actions=a0)
    assert np.allclose(r2 - r0, 0.25 * env_.normals(spec.seed, 0, 0, 3, 8).reshape(4, 2), atol=1e-6)
    noisy_tr = _env(obs_noise=0.0, reward_noise=0.0, trans_noise=0.1)
    o3, _, _, _ = env_.rollout(spec, noisy_tr, params, 0, 0, forced_actions=a0)
    zeta = env_.normals(spec.seed, 0, 0, 4, 4 * 2 * 3).reshape(4, 2, 3)
    assert np.allclose(o3[:, 1] - o0[:, 1], 0.1 * zeta[:, 0] @ quiet.C.T, atol=1e-5)     # one transition's noise, seen through C


def test_actions_come_from_the_members_policy():
    e = _env()
    spec = _spec(B=64, T=4)
    rng = np.random.default_rng(3)
    params = _params(spec, rng, scale=0.0)                            # zero network: uniform policy
    _, a, _, _ = env_.rollout(spec, e, params, 1, 0)
    assert np.all(np.bincount(a.ravel(), minlength=4) > 30)
    params[-1] = (params[-1][0], np.array([0.0, 30.0, 0.0, 0.0, 0.0]))   # a bias that always picks action 1
    _, a, _, margin = env_.rollout(spec, e, params, 1, 0)
    assert np.all(a == 1) and np.all(margin > 1e-6)
    # forcing other actions changes the states but not what the policy itself would have chosen at time 0
    forced = np.full_like(a, 2)
    o2, a2, _, _ = env_.rollout(spec, e, params, 1, 0, forced_actions=forced)
    assert np.all(a2 == 1)


def test_return_depends_on_the_policy():
    """The score (mean return) of a member that prefers the action pushing the latent along w beats the
    score of one that prefers the opposite action: `eval` is a function of theta."""
    nz, na, d = 3, 4, 6
    w = np.array([1.0, 0.0, 0.0])
    Bm = np.zeros((nz, na))
    Bm[0, 0], Bm[0, 1] = 1.0, -1.0
    e = env_.Environment(0.5 * np.eye(nz), Bm, np.random.default_rng(0).standard_normal((d, nz)), w)
    spec = _spec(B=32, T=10)
    good = _params(spec, np.random.default_rng(1), scale=0.0)
    bad = _params(spec, np.random.default_rng(1), scale=0.0)
    good[-1] = (good[-1][0], np.array([5.0, 0.0, 0.0, 0.0, 0.0]))
    bad[-1] = (bad[-1][0], np.array([0.0, 5.0, 0.0, 0.0, 0.0]))
    ret = lambda p: float(env_.rollout(spec, e, p, 0, 0)[2].astype(np.float64).sum(axis=1).mean())
    assert ret(good) > ret(bad) + 5.0


def test_step_on_policy_uses_the_generated_unroll():
    e = _env()
    spec = _spec(B=6, T=3)
    rng = np.random.default_rng(4)
    layers = _params(spec, rng)
    m1 = a2c.new_member(spec, layers, np.array([1e-3, 1e-2], dtype=np.float32), 0)
    m2 = a2c.new_member(spec, layers, np.array([1e-3, 1e-2], dtype=np.float32), 0)
    loss1, batch = a2c.step_on_policy(spec, e, m1, 0, 3)
    obs, actions, rewards, _ = env_.rollout(spec, e, a2c.params_of(m2), 0, 3)
    loss2, _ = a2c.step_on_policy(spec, e, m2, 0, 3, batch=(obs, actions, rewards))
    assert loss1 == loss2 and all(np.array_equal(a, b) for a, b in zip(m1.theta, m2.theta))
    assert m1.hist == [np.float32(rewards.astype(np.float64).sum(axis=1).mean())] and m1.t == 1
    assert a2c.evaluate(spec, m1) == m1.hist[0]
