"""Workload definitions and seeded synthetic inputs.

This module holds no arithmetic of the method: it only names shapes and
constants of the synthetic workloads and draws their inputs (data sets,
initial weights, initial hyperparameters) from numpy's seeded generator.  The
same arrays are handed to the GPU library and to whatever they are checked
against, so input generation is never a surface on which the two can differ.

The workloads stand in for the paper's experiments (Section 4), whose data sets
and environments are not redistributable with a benchmark: Gaussian-mixture
classifiers for generic supervised learning (Section 3), an MLP GAN for the
CIFAR GAN of Section 4.3, a small decoder-only transformer for the translation
model of Section 4.2 and an actor-critic MLP for the agents of Section 4.1.
"""
import math
import numpy as np

ACT_NONE, ACT_RELU, ACT_GELU, ACT_LEAKY_RELU, ACT_TANH = 0, 1, 2, 3, 4
OPT_SGD_MOMENTUM, OPT_ADAM, OPT_RMSPROP = 0, 1, 2
DTYPE_FP32, DTYPE_BF16 = 0, 1
ROLE_LR, ROLE_BETA1, ROLE_WD, ROLE_LR_G, ROLE_LR_D, ROLE_ENTROPY_COST, ROLE_DROPOUT, ROLE_LABEL_SMOOTH = 0, 1, 2, 3, 4, 5, 6, 7
WL_CLASSIFIER, WL_GAN, WL_TRANSFORMER, WL_A2C = 1, 3, 4, 5

POPULATION_SEED = 2017          # Philox key of the population


def trunc_count(P, percent):
    """Size of the top and of the bottom set: floor(P * percent / 100), at least 1."""
    return max(1, (P * percent) // 100)


class Workload:
    def __init__(self, **kw):
        self.__dict__.update(kw)

    def replace(self, **kw):
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)


# Two-layer fp32 MLPs, SGD with momentum; lr is the one hyperparameter.
MLP_SMALL = Workload(
    name="mlp_small_fp32", kind=WL_CLASSIFIER, P=8, dims=[32, 64, 4], act=ACT_RELU,
    dtype=DTYPE_FP32, optimizer=OPT_SGD_MOMENTUM, batch=64, n_train=4096, n_eval=1024,
    n_classes=4, roles=[ROLE_LR], priors=[("log", 1e-3, 1e-1)], h_max=[math.inf],
    ready_interval=50, n_trunc=trunc_count(8, 25), total_steps=1000,
    opt_const=dict(momentum=0.9), data_seed=1001, perturb=(0.8, 1.2))

# bf16 MLPs with fp32 master weights, Adam; lr, beta1 and weight decay per member.
MLP_WIDE = Workload(
    name="mlp_wide_bf16", kind=WL_CLASSIFIER, P=64, dims=[256, 1024, 1024, 10], act=ACT_GELU,
    dtype=DTYPE_BF16, optimizer=OPT_ADAM, batch=128, n_train=65536, n_eval=8192,
    n_classes=10, roles=[ROLE_LR, ROLE_BETA1, ROLE_WD],
    priors=[("log", 1e-4, 1e-2), ("uniform", 0.8, 0.95), ("log", 1e-6, 1e-3)],
    h_max=[math.inf, 0.999, math.inf],
    ready_interval=200, n_trunc=trunc_count(64, 20), total_steps=10000,
    opt_const=dict(beta2=0.999, eps=1e-8), data_seed=1002, perturb=(0.8, 1.2))

# MLP GAN pairs: generator latent -> data (tanh), discriminator data -> logit (LeakyReLU 0.2); Adam with
# beta1 0.5 (the paper's GAN appendix), separate generator / discriminator learning rates per member.
GAN_MLP = Workload(
    name="gan_mlp_bf16", kind=WL_GAN, P=32, dims=[128, 512, 512, 784], act=ACT_RELU, act_out=ACT_TANH,
    dims2=[784, 512, 512, 1], act2=ACT_LEAKY_RELU, dtype=DTYPE_BF16, optimizer=OPT_ADAM, batch=64,
    n_train=65536, n_eval=2048, roles=[ROLE_LR_G, ROLE_LR_D], priors=[("log", 1e-5, 1e-3), ("log", 1e-5, 1e-3)],
    h_max=[math.inf, math.inf], ready_interval=500, n_trunc=trunc_count(32, 20), total_steps=20000,
    opt_const=dict(beta1=0.5, beta2=0.999, eps=1e-8), data_seed=1003, perturb=(0.8, 1.2),
    n_modes=16, rank=32)

# The same pairs trained as in the paper's GAN experiment (Section 4.3.1): 5 critic updates per generator update
# on the WGAN-GP objective, perturb factors 2.0 / 0.5.
GAN_MLP_WGAN_GP = GAN_MLP.replace(objective="wgan_gp", n_critic=5, gp_weight=10.0, perturb=(0.5, 2.0))

# Actor-critic MLP agents on pre-recorded synthetic trajectories: torso 512-256-256 (ReLU), one head with 18
# policy logits + 1 value; RMSProp; learning rate and entropy cost per member; 32 trajectories of 20
# transitions per step; score = mean of the last 10 unroll returns.
A2C_MLP = Workload(
    name="a2c_mlp_bf16", kind=WL_A2C, P=128, dims=[512, 256, 256, 19], act=ACT_RELU, dtype=DTYPE_BF16,
    optimizer=OPT_RMSPROP, batch=32, unroll=20, gamma=0.99, value_cost=0.5, n_actions=18, latent=16,
    n_train=4096, n_eval=1, roles=[ROLE_LR, ROLE_ENTROPY_COST], priors=[("log", 1e-5, 1e-3), ("log", 1e-4, 1e-2)],
    h_max=[math.inf, math.inf], ready_interval=100, n_trunc=trunc_count(128, 20), total_steps=2000,
    opt_const=dict(rho=0.99, eps=1e-5), data_seed=1005, perturb=(0.8, 1.2))

# The same agents acting with their current policy: every step generates its unroll on the device in the
# latent system of latent_system() (the score then depends on the member's weights).
A2C_MLP_ON_POLICY = A2C_MLP.replace(on_policy=1)

# Decoder-only transformers (pre-LayerNorm blocks, learned positions, untied head) on synthetic token
# sequences; Adam; learning rate, one dropout rate and the label smoothing per member; score = minus the
# held-out perplexity.
TRANSFORMER = Workload(
    name="transformer_bf16", kind=WL_TRANSFORMER, P=16, vocab=8192, d_model=512, heads=8, d_ff=2048, n_blocks=4,
    seq=128, batch=32, dtype=DTYPE_BF16, optimizer=OPT_ADAM, act=ACT_RELU, dims=[], n_train=8192, n_eval=256,
    roles=[ROLE_LR, ROLE_DROPOUT, ROLE_LABEL_SMOOTH],
    priors=[("log", 1e-4, 1e-3), ("uniform", 0.0, 0.3), ("uniform", 0.0, 0.2)], h_max=[math.inf, 0.9, 0.9],
    ready_interval=200, n_trunc=trunc_count(16, 20), total_steps=2000,
    opt_const=dict(beta1=0.9, beta2=0.999, eps=1e-8), data_seed=1004, perturb=(0.8, 1.2), zipf_s=1.1)

WORKLOADS = {1: MLP_SMALL, 2: MLP_WIDE, 3: GAN_MLP, 4: TRANSFORMER, 5: A2C_MLP}


def transformer_shapes(wl):
    """Shapes of the parameter arrays of one transformer, in the order of the flat parameter vector."""
    d, f, V, S = wl.d_model, wl.d_ff, wl.vocab, wl.seq
    out = [(V, d), (S, d)]
    for _ in range(wl.n_blocks):
        out += [(d,), (d,), (d, 3 * d), (3 * d,), (d, d), (d,), (d,), (d,), (d, f), (f,), (f, d), (d,)]
    return out + [(d,), (d,), (d, V), (V,)]


def initial_transformer_weights(wl, P, seed):
    """Per member the parameter arrays in layout order: embeddings ~ N(0, 0.1^2), matrices uniform in
    +-1/sqrt(fan_in), LayerNorm gains 1, every bias 0."""
    rng = np.random.default_rng(seed)
    shapes = transformer_shapes(wl)
    gains = {2 + 12 * l + k for l in range(wl.n_blocks) for k in (0, 6)} | {len(shapes) - 4}
    members = []
    for _ in range(P):
        arrays = []
        for j, sh in enumerate(shapes):
            if j < 2:
                arrays.append((0.1 * rng.standard_normal(sh)).astype(np.float32))
            elif len(sh) == 2:
                lim = 1.0 / math.sqrt(sh[0])
                arrays.append(rng.uniform(-lim, lim, size=sh).astype(np.float32))
            else:
                arrays.append(np.full(sh, 1.0 if j in gains else 0.0, dtype=np.float32))
        members.append(arrays)
    return members


def zipf_bigram_sequences(wl):
    """(train [n_train][seq+1], eval [n_eval][seq+1]) int32 token sequences.  Ranks z_t are i.i.d. from a
    Zipf(s) law truncated to the vocabulary (inverse-CDF lookup); with a fixed random permutation pi of
    the vocabulary, x_0 = z_0 - 1 and x_t = (pi[x_{t-1}] + z_t - 1) mod V, so the next token is
    predictable from the current one up to the entropy of the Zipf law."""
    rng = np.random.default_rng(wl.data_seed)
    V, T = wl.vocab, wl.seq + 1
    pmf = 1.0 / np.arange(1, V + 1) ** wl.zipf_s
    cdf = np.cumsum(pmf / pmf.sum())
    pi = rng.permutation(V)
    out = []
    for n in (wl.n_train, wl.n_eval):
        z = np.minimum(np.searchsorted(cdf, rng.random((n, T))), V - 1)      # rank - 1
        x = np.empty((n, T), dtype=np.int64)
        x[:, 0] = z[:, 0]
        for t in range(1, T):
            x[:, t] = (pi[x[:, t - 1]] + z[:, t]) % V
        out.append(x.astype(np.int32))
    return out[0], out[1]


def gaussian_mixture(n_classes, dim, n_train, n_eval, seed):
    """Class means ~ N(0, I); x = mean[label] + N(0, I); labels uniform."""
    rng = np.random.default_rng(seed)
    means = rng.standard_normal((n_classes, dim))
    out = []
    for n in (n_train, n_eval):
        y = rng.integers(0, n_classes, size=n).astype(np.int32)
        x = (means[y] + rng.standard_normal((n, dim))).astype(np.float32)
        out.append((x, y))
    return out[0], out[1]


def classifier_data(wl):
    return gaussian_mixture(wl.n_classes, wl.dims[0], wl.n_train, wl.n_eval, wl.data_seed)


def low_rank_mixture(n_modes, dim, rank, n_train, n_eval, seed):
    """x = mu_k + A_k e with k uniform over the modes, e ~ N(0, I_rank), A_k ~ N(0, 1) * 0.25 / sqrt(rank),
    mu_k ~ N(0, 0.25^2 I): a mixture of low-rank Gaussians that fits the range of a tanh output."""
    rng = np.random.default_rng(seed)
    mu = rng.standard_normal((n_modes, dim)) * 0.25
    A = rng.standard_normal((n_modes, dim, rank)) * (0.25 / math.sqrt(rank))
    out = []
    for n in (n_train, n_eval):
        k = rng.integers(0, n_modes, size=n)
        e = rng.standard_normal((n, rank))
        x = mu[k] + np.einsum("ndr,nr->nd", A[k], e)
        out.append(x.astype(np.float32))
    return out[0], out[1]


def gan_data(wl):
    return low_rank_mixture(wl.n_modes, wl.dims2[0], wl.rank, wl.n_train, wl.n_eval, wl.data_seed)


def initial_gan_weights(wl, P, seed):
    """Per member: (generator layers, discriminator layers)."""
    g = initial_mlp_weights(wl.dims, P, seed)
    d = initial_mlp_weights(wl.dims2, P, seed + 1000)
    return [(g[i], d[i]) for i in range(P)]


def latent_system(wl):
    """The linear-Gaussian latent system of the actor-critic workload, from the data seed:
    A = 0.9 x random orthogonal [n_z][n_z], B ~ N(0, 0.3^2) [n_z][n_actions], C ~ N(0, 1) / 4 [d][n_z],
    reward direction w ~ N(0, 1) [n_z]; float64 arrays.  (The same draws, in the same order, that
    trajectory_pool starts with.)"""
    rng = np.random.default_rng(wl.data_seed)
    nz, d = wl.latent, wl.dims[0]
    Q, _ = np.linalg.qr(rng.standard_normal((nz, nz)))
    A = 0.9 * Q
    Bm = rng.standard_normal((nz, wl.n_actions)) * 0.3
    C = rng.standard_normal((d, nz)) / 4.0
    w = rng.standard_normal(nz)
    return A, Bm, C, w


def trajectory_pool(wl):
    """Pre-recorded trajectories from a linear-Gaussian latent system with uniformly random actions:
    z' = A z + B e(a) + 0.1 xi (A = 0.9 x random orthogonal, B ~ N(0, 0.3^2)), observation = C z + N(0, I)
    (C ~ N(0, 1) / 4), reward = w.z + 0.1 noise.  Returns (obs [n][T+1][d], actions [n][T], rewards [n][T])."""
    rng = np.random.default_rng(wl.data_seed)
    nz, d, T, n = wl.latent, wl.dims[0], wl.unroll, wl.n_train
    Q, _ = np.linalg.qr(rng.standard_normal((nz, nz)))
    A = 0.9 * Q
    Bm = rng.standard_normal((nz, wl.n_actions)) * 0.3
    C = rng.standard_normal((d, nz)) / 4.0
    w = rng.standard_normal(nz)
    z = rng.standard_normal((n, nz))
    obs = np.empty((n, T + 1, d), dtype=np.float32)
    actions = rng.integers(0, wl.n_actions, size=(n, T)).astype(np.int32)
    rewards = np.empty((n, T), dtype=np.float32)
    for t in range(T + 1):
        obs[:, t] = z @ C.T + rng.standard_normal((n, d))
        if t < T:
            rewards[:, t] = z @ w + 0.1 * rng.standard_normal(n)
            z = z @ A.T + Bm[:, actions[:, t]].T + 0.1 * rng.standard_normal((n, nz))
    return obs, actions, rewards


def initial_hypers(wl, seed):
    """float32 array [P][n_h] drawn from the priors ("log" = log-uniform)."""
    rng = np.random.default_rng(seed)
    H = np.empty((wl.P, len(wl.priors)), dtype=np.float32)
    for k, (kind, lo, hi) in enumerate(wl.priors):
        u = rng.random(wl.P)
        if kind == "log":
            H[:, k] = np.exp(math.log(lo) + u * (math.log(hi) - math.log(lo)))
        else:
            H[:, k] = lo + u * (hi - lo)
    return H


def initial_mlp_weights(dims, P, seed):
    """Per member a list of (W[fan_in][fan_out], b[fan_out]) float32 arrays,
    uniform in +-1/sqrt(fan_in)."""
    rng = np.random.default_rng(seed)
    pop = []
    for _ in range(P):
        layers = []
        for fi, fo in zip(dims[:-1], dims[1:]):
            bound = 1.0 / math.sqrt(fi)
            W = rng.uniform(-bound, bound, size=(fi, fo)).astype(np.float32)
            b = rng.uniform(-bound, bound, size=(fo,)).astype(np.float32)
            layers.append((W, b))
        pop.append(layers)
    return pop
