"""On-policy unrolls for the actor-critic workload (oracle side).

The paper's reinforcement-learning agents (Section 4.1.1) act in their environment with their current
policy, and `eval` is the mean of the last 10 episodic returns, so a member's score depends on its
weights.  This synthetic stand-in generates every unroll from the member's current policy in a
linear-Gaussian latent system:

    z_0 ~ N(0, I)                                   latent state, dimension n_z
    o_t = C z_t + obs_noise * xi_t                  observation, xi ~ N(0, I_d), stored as float32
    a_t ~ softmax(policy logits of the member's network on o_t)
    r_t = w . z_t + reward_noise * nu_t             stored as float32
    z_{t+1} = A z_t + B[:, a_t] + trans_noise * zeta_t

for t = 0 .. T-1, plus the observation o_T that the value bootstrap needs.  The environment (A, B, C, w
and the three noise scales) is an input, the same for every member.

Random numbers (Philox counter (step, member, domain, e // 4), element e of a stream):
    DOMAIN_ENV + 0  z_0,   e = r * n_z + k            standard normal
    DOMAIN_ENV + 1  xi,    e = (r * (T+1) + t) * d + j  standard normal
    DOMAIN_ENV + 2  u,     counter element r * T + t, word 0: u = (x + 0.5) / 2^32
    DOMAIN_ENV + 3  nu,    e = r * T + t              standard normal
    DOMAIN_ENV + 4  zeta,  e = (r * T + t) * n_z + k  standard normal
Normals are Box-Muller pairs: words (0, 1) and (2, 3) of a counter give one pair each, element e uses
pair (e % 4) // 2, cosine branch for even e, sine branch for odd e.

Action choice: with p = softmax(logits) in float64 and cdf_k = p_0 + ... + p_k, a_t is the number of k
with cdf_k <= u, capped at n_actions - 1 (the smallest action whose cdf exceeds u).  Two correct
implementations that differ in the last bits of the logits can disagree only where u lies next to an
edge of the cdf; `rollout` therefore also returns |u - nearest edge| for every choice.
"""
import numpy as np

from . import nets, philox

DOMAIN_ENV = 32


class Environment:
    def __init__(self, A, B, C, w, obs_noise=1.0, reward_noise=0.1, trans_noise=0.1):
        self.A, self.B, self.C, self.w = (np.asarray(x, dtype=np.float64) for x in (A, B, C, w))
        self.obs_noise, self.reward_noise, self.trans_noise = float(obs_noise), float(reward_noise), float(trans_noise)
        self.n_z, self.n_actions, self.d = self.A.shape[0], self.B.shape[1], self.C.shape[0]


def normals(seed, c0, member, substream, n):
    """n standard normal float64 values of stream DOMAIN_ENV + substream."""
    e = np.arange(n)
    w = philox.words(seed, c0, member, DOMAIN_ENV + substream, np.arange((n + 3) // 4))
    pair = (e % 4) // 2
    n_cos, n_sin = philox.normal_pairs(w[e // 4, 2 * pair], w[e // 4, 2 * pair + 1])
    return np.where(e % 2 == 0, n_cos, n_sin)


def uniforms(seed, c0, member, substream, n):
    return philox.unit_open(philox.words(seed, c0, member, DOMAIN_ENV + substream, np.arange(n))[:, 0])


def choose(logits, u):
    """Actions for rows of logits and uniforms u: (actions, |u - nearest cdf edge|)."""
    p = np.exp(nets.log_softmax(np.asarray(logits, dtype=np.float64)))
    cdf = np.cumsum(p, axis=-1)
    u = np.asarray(u, dtype=np.float64)[..., None]
    a = np.minimum((cdf <= u).sum(axis=-1), p.shape[-1] - 1)
    edges = cdf[..., :-1]                                    # the last edge is 1: u never reaches it
    return a, np.abs(edges - u).min(axis=-1)


def rollout(spec, env, params, member, step, forced_actions=None):
    """One unroll of B = spec.batch trajectories of T = spec.unroll transitions under the policy given
    by `params` ([(W, b), ...] of the actor-critic network, evaluated with the spec's rounding model).
    forced_actions [B][T]: the system follows these instead of the policy's own choices (which are
    still returned).  Returns obs [B][T+1][d] float32, chosen actions [B][T], rewards [B][T] float32,
    edge distances [B][T]."""
    B, T, nz, d = spec.batch, spec.unroll, env.n_z, env.d
    z = normals(spec.seed, step, member, 0, B * nz).reshape(B, nz)
    xi = normals(spec.seed, step, member, 1, B * (T + 1) * d).reshape(B, T + 1, d)
    u = uniforms(spec.seed, step, member, 2, B * T).reshape(B, T)
    nu = normals(spec.seed, step, member, 3, B * T).reshape(B, T)
    zeta = normals(spec.seed, step, member, 4, B * T * nz).reshape(B, T, nz)
    obs = np.empty((B, T + 1, d), dtype=np.float32)
    actions = np.empty((B, T), dtype=np.int64)
    rewards = np.empty((B, T), dtype=np.float32)
    margin = np.empty((B, T))
    for t in range(T + 1):
        obs[:, t] = z @ env.C.T + env.obs_noise * xi[:, t]
        if t == T:
            break
        out, _ = nets.mlp_forward(params, obs[:, t].astype(np.float64), spec.hidden_act, q=spec.q)
        actions[:, t], margin[:, t] = choose(out[:, :spec.n_actions], u[:, t])
        a = actions[:, t] if forced_actions is None else np.asarray(forced_actions)[:, t]
        rewards[:, t] = z @ env.w + env.reward_noise * nu[:, t]
        z = z @ env.A.T + env.B[:, a].T + env.trans_noise * zeta[:, t]
    return obs, actions, rewards, margin
