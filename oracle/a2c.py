"""`step` and `eval` for the actor-critic workload (oracle side).

The paper's reinforcement-learning experiments (Section 4.1.1) train A3C-style
agents with RMSProp, let PBT adapt the learning rate and the entropy cost, and
evaluate a member by its last 10 episodic rewards.  This synthetic stand-in
keeps that structure on pre-recorded trajectories:

  network   torso MLP (ReLU) -> one linear head with n_actions policy logits
            followed by one value output;
  step      B trajectories of T transitions (T + 1 observations) drawn from a
            pool (Philox domain 1, one draw per trajectory); returns are
            bootstrapped from the value of the last observation,
                R_T = V(s_T),  R_t = r_t + gamma R_{t+1}      (no gradient through R),
            advantage A_t = R_t - V(s_t) (treated as a constant in the policy
            term), and the loss is the mean over the B*T transitions of
                -A_t log pi(a_t|s_t) + 0.5 (R_t - V(s_t))^2 - entropy_cost * H(pi(.|s_t)),
            minimised by one RMSProp update with the member's learning rate;
            the member's entropy cost is its second hyperparameter;
            (`step_on_policy` generates the unroll from the member's current policy instead,
            see a2c_env.py; the update is the same);
  eval      the mean of the member's last (up to) 10 unroll returns, where an
            unroll's return is the mean over its B trajectories of the sum of
            the T rewards.  The history travels with the weights on exploit.
"""
import numpy as np

from . import nets, optim, philox, pbt

ROLE_LR, ROLE_ENTROPY_COST = 0, 5
HIST = 10


class A2CSpec:
    def __init__(self, torso_dims, n_actions, batch, unroll, seed, roles=(ROLE_LR, ROLE_ENTROPY_COST), gamma=0.99,
                 value_cost=0.5, rho=0.99, rms_eps=1e-5, hidden_act=nets.ACT_RELU, bf16_storage=False):
        self.dims = list(torso_dims) + [n_actions + 1]
        self.n_actions, self.batch, self.unroll, self.seed = n_actions, batch, unroll, seed
        self.roles, self.gamma, self.value_cost = list(roles), gamma, value_cost
        self.rho, self.rms_eps, self.hidden_act = rho, rms_eps, hidden_act
        self.q = nets.round_bf16 if bf16_storage else nets.identity


def new_member(spec, layers, h, index):
    flat = [np.array(a, dtype=np.float64) for Wb in layers for a in Wb]
    m = pbt.Member(flat, h, {"s0": [np.zeros_like(a) for a in flat]}, index)
    m.hist = []                                # unroll returns, oldest first, at most HIST kept
    return m


def params_of(m):
    return [(m.theta[2 * l], m.theta[2 * l + 1]) for l in range(len(m.theta) // 2)]


def returns(rewards, bootstrap, gamma):
    """rewards [B][T], bootstrap [B] -> R [B][T] with R_t = r_t + gamma R_{t+1}, R_T = bootstrap."""
    B, T = rewards.shape
    R = np.empty((B, T))
    nxt = np.asarray(bootstrap, dtype=np.float64)
    for t in range(T - 1, -1, -1):
        nxt = rewards[:, t] + gamma * nxt
        R[:, t] = nxt
    return R


def policy_terms(logits):
    """log pi and entropy H = -sum pi log pi per row."""
    lp = nets.log_softmax(logits)
    return lp, -(np.exp(lp) * lp).sum(axis=-1)


def loss_and_grads(spec, m, obs, actions, rewards):
    """obs [B][T+1][d], actions [B][T] ints, rewards [B][T].  Returns (loss, grads)."""
    B, T = actions.shape
    ent_cost = float(m.h[spec.roles.index(ROLE_ENTROPY_COST)])
    x = np.asarray(obs, dtype=np.float64).reshape(B * (T + 1), -1)
    out, cache = nets.mlp_forward(params_of(m), x, spec.hidden_act, q=spec.q)
    out = out.reshape(B, T + 1, -1)
    logits, value = out[:, :T, :spec.n_actions], out[:, :, spec.n_actions]
    R = returns(np.asarray(rewards, dtype=np.float64), value[:, T], spec.gamma)      # constants from here on
    adv = R - value[:, :T]
    lp, ent = policy_terms(logits)
    lp_a = np.take_along_axis(lp, np.asarray(actions)[..., None], axis=-1)[..., 0]
    n = B * T
    loss = (-(adv * lp_a).sum() + spec.value_cost * ((R - value[:, :T]) ** 2).sum() - ent_cost * ent.sum()) / n
    # gradient with respect to the head's outputs
    pi = np.exp(lp)
    onehot = np.zeros_like(pi)
    np.put_along_axis(onehot, np.asarray(actions)[..., None], 1.0, axis=-1)
    d_logits = (-adv[..., None] * (onehot - pi) + ent_cost * pi * (lp + ent[..., None])) / n
    d_value = 2.0 * spec.value_cost * (value[:, :T] - R) / n
    d_out = np.zeros_like(out)
    d_out[:, :T, :spec.n_actions] = d_logits
    d_out[:, :T, spec.n_actions] = d_value                   # the bootstrap row gets no gradient
    grads, _ = nets.mlp_backward(params_of(m), cache, d_out.reshape(B * (T + 1), -1), spec.hidden_act, q=spec.q)
    return loss, grads


def update_on_batch(spec, m, obs, actions, rewards):
    """One RMSProp update on a given unroll; pushes the unroll's return onto the member's history."""
    loss, grads = loss_and_grads(spec, m, obs, actions, rewards)
    lr = m.h[spec.roles.index(ROLE_LR)]
    m.t += 1
    for j, g in enumerate([a for gr in grads for a in gr]):
        m.theta[j], m.opt["s0"][j] = optim.rmsprop(m.theta[j], g, m.opt["s0"][j], lr, spec.rho, spec.rms_eps)
    # float32 like the population store keeps it
    m.hist = (m.hist + [np.float32(np.asarray(rewards, dtype=np.float64).sum(axis=1).mean())])[-HIST:]
    return loss


def step(spec, m, i, s, pool_obs, pool_actions, pool_rewards):
    """`step` on pre-recorded trajectories: B draws from the pool (Philox domain 1, one per trajectory)."""
    idx = philox.bounded(philox.words(spec.seed, s, i, philox.DOMAIN_BATCH, np.arange(spec.batch))[..., 0], len(pool_obs))
    return update_on_batch(spec, m, pool_obs[idx], pool_actions[idx], pool_rewards[idx])


def step_on_policy(spec, env, m, i, s, batch=None):
    """`step` on an unroll generated from the member's current policy (a2c_env.rollout), or on a given
    batch = (obs, actions, rewards) that such a generator produced.  Returns (loss, batch)."""
    from . import a2c_env
    if batch is None:
        batch = a2c_env.rollout(spec, env, params_of(m), i, s)[:3]
    return update_on_batch(spec, m, *batch), batch


def evaluate(spec, m):
    """`eval`: mean of the last (up to) 10 unroll returns; -inf before the first step."""
    if not m.hist:
        return np.float32(-np.inf)
    return np.float32(np.mean(np.asarray(m.hist, dtype=np.float64)))
