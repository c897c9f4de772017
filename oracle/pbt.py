"""Population Based Training: the population store and the exploit/explore
pass, in the synchronous form (oracle side).

Follows Algorithm 1 of the paper (Section 3) executed with the partial
synchrony of Appendix A.1: every member is advanced by `step` for a fixed
number of iterations, then `eval` scores every member and the
exploit-and-explore procedure runs over the whole population, and the cycle
repeats.  `exploit` is truncation selection by default (Section 4.1.1, Exploit (b)): rank
all members by score; each member of the bottom set samples a donor uniformly
from the top set and takes over its weights and hyperparameters.  `explore` is
perturb (Section 4.1.1, Explore (a)): every hyperparameter of a member that was
overwritten is multiplied, independently, by one of two factors.  Members that
were not overwritten are left exactly as they were (the `theta != theta'`
test of Algorithm 1).

Readings where the paper is silent (kept identical, as text, on the GPU side):
  * the sizes of top and bottom set are one integer `n_trunc`, 2 n_trunc <= P;
  * order = score descending, ties by lower member index first, -inf after
    every finite score, NaN after -inf;
  * donors are drawn independently per recipient (with replacement) from one
    Philox word: top[(x * n_trunc) >> 32];
  * factor = low bit of a Philox word: 0 -> lower factor, 1 -> upper factor;
  * the multiply is an IEEE float32 multiply of the donor's float32
    hyperparameter by the float32-rounded factor, followed by an upper clamp
    for hyperparameters that are probabilities (no clamp to the prior range);
  * the optimiser state and the update count are copied with the weights, and
    so are the donor's score and score history (re-evaluating a byte-identical
    copy, as Algorithm 1 does after explore, would return the same number).
"""
import copy
import math
import numpy as np

from . import philox


class Member:
    """One tuple (theta, h, p, t) of the population, plus optimiser state and
    the index of the member it last copied from."""

    def __init__(self, theta, h, opt_state=None, index=0):
        self.theta = theta                        # list of float64 arrays
        self.opt = opt_state if opt_state is not None else {}
        self.h = np.asarray(h, dtype=np.float32).copy()
        self.p = np.float32(-np.inf)
        self.t = 0                                # optimiser updates applied
        self.parent = index
        self.hist = None                          # optional score history


def init_hyperparameters(seed, P, priors):
    """Initial h (Figure 1c: hyperparameters are sampled at random to start with): column k of
    member i is drawn from priors[k] = (kind, lo, hi), kind "uniform" or "log" (log-uniform:
    exp of a uniform draw between ln lo and ln hi), using u = (x + 0.5) / 2**32 with x word 0 of
    Philox counter (0, i, DOMAIN_INIT_H, k).  Returned as float32 [P][n_h]."""
    H = np.empty((P, len(priors)), dtype=np.float32)
    for k, (kind, lo, hi) in enumerate(priors):
        x = philox.words(seed, 0, np.arange(P), philox.DOMAIN_INIT_H, k)[:, 0]
        u = philox.unit_open(x)
        if kind == "log":
            H[:, k] = np.exp(math.log(lo) + u * (math.log(hi) - math.log(lo)))
        elif kind == "uniform":
            H[:, k] = lo + u * (hi - lo)
        else:
            raise ValueError(kind)
    return H


def init_weights(seed, member, dims, offsets):
    """Initial theta of one member (Figure 1c: random weight initialisations): every weight and
    bias of a layer with fan-in f is uniform in (-1/sqrt f, 1/sqrt f).  The value at position p
    of the member's flat parameter vector uses word p % 4 of Philox counter
    (0, member, DOMAIN_INIT_W, p // 4); offsets[l] = (start of W_l, start of b_l) in that vector.
    Returns [(W, b), ...] rounded to float32."""
    layers = []
    for l, (fi, fo) in enumerate(zip(dims[:-1], dims[1:])):
        out = []
        for start, count in ((offsets[l][0], fi * fo), (offsets[l][1], fo)):
            pos = start + np.arange(count)
            w = philox.words(seed, 0, member, philox.DOMAIN_INIT_W, pos // 4)
            x = w[np.arange(count), pos % 4]
            u = philox.unit_open(x)
            out.append(((2.0 * u - 1.0) / math.sqrt(fi)).astype(np.float32))
        layers.append((out[0].reshape(fi, fo), out[1]))
    return layers


def init_segments(seed, member, segments):
    """Initial values of arbitrary parameter arrays of one member: segments = [(start, shape, fan,
    const), ...] in positions of the member's flat vector; fan > 0: uniform in (-1/sqrt fan, 1/sqrt fan)
    from the same Philox words as init_weights (word p % 4 of counter (0, member, DOMAIN_INIT_W,
    p // 4) for position p); fan == 0: the constant.  Returns float32 arrays."""
    out = []
    for start, shape, fan, const in segments:
        count = int(np.prod(shape))
        if fan > 0:
            pos = start + np.arange(count)
            w = philox.words(seed, 0, member, philox.DOMAIN_INIT_W, pos // 4)
            u = philox.unit_open(w[np.arange(count), pos % 4])
            out.append(((2.0 * u - 1.0) / math.sqrt(fan)).astype(np.float32).reshape(shape))
        else:
            out.append(np.full(shape, const, dtype=np.float32))
    return out


def rank_order(scores):
    """Member indices from best to worst."""
    s = np.asarray(scores, dtype=np.float32)

    def key(i):
        v = float(s[i])
        if math.isnan(v):
            return (1, 0.0, i)
        return (0, -v, i)
    return sorted(range(len(s)), key=key)


def truncation_select(scores, n_trunc, round_index, seed):
    """Returns (order, donor): donor[i] = member i copies from, or -1."""
    P = len(scores)
    if not 0 <= 2 * n_trunc <= P:
        raise ValueError("need 0 <= 2*n_trunc <= P")
    order = rank_order(scores)
    donor = np.full(P, -1, dtype=np.int32)
    if n_trunc == 0:
        return order, donor
    top = order[:n_trunc]
    bottom = order[P - n_trunc:]
    for r in bottom:
        x = philox.words(seed, round_index, r, philox.DOMAIN_DONOR, 0)[0]
        donor[r] = top[int(philox.bounded(x, n_trunc))]
    return order, donor


def binary_tournament(scores, round_index, seed):
    """Section 4.3.1, Exploit (b): every member draws ONE other member uniformly at random and copies
    it if the other member's score is better.  "Better" is the total order of rank_order (so NaN and
    -inf members always lose, ties go to the lower index).  Opponent of member i: j = floor(x (P-1) /
    2^32) from word 0 of Philox counter (round, i, DOMAIN_DONOR, 0), then j += 1 if j >= i (uniform
    over the P-1 others).  All members decide on the scores as they were before the pass.
    Returns (order, donor): donor[i] = member i copies from, or -1."""
    P = len(scores)
    order = rank_order(scores)
    place = np.empty(P, dtype=np.int64)
    place[order] = np.arange(P)
    donor = np.full(P, -1, dtype=np.int32)
    if P < 2:
        return order, donor
    for i in range(P):
        x = philox.words(seed, round_index, i, philox.DOMAIN_DONOR, 0)[0]
        j = int(philox.bounded(x, P - 1))
        j += 1 if j >= i else 0
        if place[j] < place[i]:
            donor[i] = j
    return order, donor


def student_sf(t, nu):
    """P(T > t) for Student's t distribution with nu degrees of freedom, t >= 0:
    half the regularised incomplete beta function I_x(nu/2, 1/2) at x = nu / (nu + t^2)."""
    from scipy.special import betainc
    return 0.5 * float(betainc(0.5 * nu, 0.5, nu / (nu + t * t)))


def welch(a, b):
    """Welch's unequal-variance statistic for "mean(b) > mean(a)": returns (t, nu, mean_a, mean_b) with
    t = (mean_b - mean_a) / sqrt(va + vb), v = s^2 / n (s^2 the unbiased sample variance), and the
    Welch-Satterthwaite degrees of freedom nu = (va + vb)^2 / (va^2/(na-1) + vb^2/(nb-1)).
    t = nu = inf when both variances are zero."""
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    na, nb = len(a), len(b)
    ma, mb = a.sum() / na, b.sum() / nb
    va = ((a - ma) ** 2).sum() / (na - 1) / na
    vb = ((b - mb) ** 2).sum() / (nb - 1) / nb
    if va + vb == 0.0:
        return math.inf, math.inf, ma, mb
    t = (mb - ma) / math.sqrt(va + vb)
    nu = (va + vb) ** 2 / (va * va / (na - 1) + vb * vb / (nb - 1))
    return t, nu, ma, mb


def ttest_select(scores, hists, round_index, seed, alpha):
    """Section 4.1.1, Exploit (a): every member draws one other member uniformly (as in the binary
    tournament) and copies it if that member's recent scores (hists[j], oldest first, the last up to
    10 evaluations) have a higher mean than its own AND Welch's t-test rejects equality of the means in
    that direction at level alpha (one-sided p < alpha; zero variance on both sides counts as
    rejected).  Members with fewer than two recorded scores neither copy nor get copied.
    Returns (order, donor)."""
    P = len(scores)
    order = rank_order(scores)
    donor = np.full(P, -1, dtype=np.int32)
    if P < 2:
        return order, donor
    for i in range(P):
        x = philox.words(seed, round_index, i, philox.DOMAIN_DONOR, 0)[0]
        j = int(philox.bounded(x, P - 1))
        j += 1 if j >= i else 0
        if hists[i] is None or hists[j] is None or len(hists[i]) < 2 or len(hists[j]) < 2:
            continue
        t, nu, mi, mj = welch(hists[i], hists[j])
        if mj > mi and (math.isinf(t) or student_sf(t, nu) < alpha):
            donor[i] = j
    return order, donor


def resample(h_src, round_index, r, seed, prob, priors, h_max=None):
    """Explore (b) of Section 4.1.1 for recipient r: every hyperparameter is, independently and with
    probability `prob`, drawn afresh from its prior (kind, lo, hi); otherwise the copied value is kept.
    Hyperparameter k uses Philox counter (round, r, DOMAIN_EXPLORE, k): resample iff word 1 <
    floor(prob 2^32) (prob >= 1: always), new value = prior map of u = (word 2 + 0.5) / 2^32, computed
    in double and rounded to float32 as for the initial population."""
    h_src = np.asarray(h_src, dtype=np.float32)
    out = h_src.copy()
    thr = int(math.floor(float(np.float32(prob)) * 4294967296.0))
    for k, (kind, lo, hi) in enumerate(priors):
        w = philox.words(seed, round_index, r, philox.DOMAIN_EXPLORE, k)
        if prob >= 1.0 or int(w[1]) < thr:
            u = float(philox.unit_open(w[2]))
            if kind == "log":
                v = np.float32(math.exp(math.log(lo) + u * (math.log(hi) - math.log(lo))))
            elif kind == "uniform":
                v = np.float32(lo + u * (hi - lo))
            else:
                raise ValueError(kind)
            out[k] = v
        if h_max is not None and out[k] > np.float32(h_max[k]):
            out[k] = np.float32(h_max[k])
    return out


def perturb(h_src, round_index, r, seed, factor_lo, factor_hi, h_max=None):
    """Explore for recipient r: float32 multiply of every hyperparameter of the
    source vector by factor_lo or factor_hi."""
    h_src = np.asarray(h_src, dtype=np.float32)
    out = np.empty_like(h_src)
    f_lo = np.float32(factor_lo)
    f_hi = np.float32(factor_hi)
    for k in range(len(h_src)):
        bit = int(philox.words(seed, round_index, r, philox.DOMAIN_EXPLORE, k)[0]) & 1
        f = f_hi if bit else f_lo
        # product of two float32 values is exact in float64; one rounding to
        # float32 is the IEEE float32 multiply
        v = np.float32(np.float64(h_src[k]) * np.float64(f))
        if h_max is not None and v > np.float32(h_max[k]):
            v = np.float32(h_max[k])
        out[k] = v
    return out


def exploit_explore(pop, round_index, seed, n_trunc, factor_lo=0.8, factor_hi=1.2, h_max=None,
                    scores=None, explore_fn=None, mode="truncation", copy_weights=True, copy_hypers=True,
                    explore="perturb", resample_prob=0.0, priors=None, ttest_alpha=0.05):
    """One exploit-and-explore pass over the population, in place.
    `scores` overrides the members' stored p (float32).  `explore_fn(h, round,
    r)` replaces the explore rule (used by the toy example).  Returns (order, donor).

    mode: "truncation" (Section 4.1.1 Exploit (b)), "tournament" (Section 4.3.1 Exploit (b)) or "ttest"
    (Section 4.1.1 Exploit (a), on the members' score histories).  In the last two a member can be donor
    and recipient in the same pass; every recipient receives its
    donor's state as it was BEFORE the pass (all members act on the same snapshot).
    copy_weights / copy_hypers: the subsets of Section 4.4 ("PBT targets"): without copy_weights the
    recipient keeps its own weights, optimiser state, update count, score and history and only takes
    (explored) hyperparameters; without copy_hypers it takes the weights and keeps its own
    hyperparameters, which are then neither copied nor explored.
    explore: "perturb" (Section 4.1.1 Explore (a)) or "resample" (Explore (b), needs priors)."""
    if scores is None:
        scores = np.array([m.p for m in pop], dtype=np.float32)
    else:
        scores = np.asarray(scores, dtype=np.float32)
        for m, s in zip(pop, scores):
            m.p = np.float32(s)
    if mode == "truncation":
        order, donor = truncation_select(scores, n_trunc, round_index, seed)
    elif mode == "tournament":
        order, donor = binary_tournament(scores, round_index, seed)
    elif mode == "ttest":
        order, donor = ttest_select(scores, [m.hist for m in pop], round_index, seed, ttest_alpha)
    else:
        raise ValueError(mode)
    # assignments below replace attributes and never change the old objects, so these references are a snapshot
    before = [(m.theta, m.opt, m.t, m.p, m.hist, m.h) for m in pop]
    for r in range(len(pop)):
        d = int(donor[r])
        if d < 0:
            continue
        theta, opt, t, p, hist, h = before[d]
        dst = pop[r]
        if copy_weights:
            dst.theta = copy.deepcopy(theta)
            dst.opt = copy.deepcopy(opt)
            dst.t = t
            dst.p = p
            dst.hist = copy.deepcopy(hist)
        if copy_hypers:
            if explore_fn is not None:
                dst.h = np.asarray(explore_fn(h, round_index, r), dtype=np.float32)
            elif explore == "perturb":
                dst.h = perturb(h, round_index, r, seed, factor_lo, factor_hi, h_max)
            elif explore == "resample":
                dst.h = resample(h, round_index, r, seed, resample_prob, priors, h_max)
            else:
                raise ValueError(explore)
        dst.parent = d
    return order, donor


def train(pop, n_steps, step_fn, eval_fn, ready_interval, exploit_explore_fn, log=None):
    """Algorithm 1 in lock-step.  step_fn(member, i, s) applies one update,
    eval_fn(member, i) returns the score, exploit_explore_fn(pop, round) runs
    the pass.  Returns the index of the member with the highest score."""
    round_index = 0
    for s in range(n_steps):
        for i, m in enumerate(pop):
            step_fn(m, i, s)
        if ready_interval > 0 and (s + 1) % ready_interval == 0:
            for i, m in enumerate(pop):
                m.p = np.float32(eval_fn(m, i))
            res = exploit_explore_fn(pop, round_index)
            if log is not None:
                log(s, round_index, res)
            round_index += 1
    for i, m in enumerate(pop):
        m.p = np.float32(eval_fn(m, i))
    return rank_order([m.p for m in pop])[0]


# ----------------------------------------------------------------------------
# The toy example of Figure 2: maximise Q(theta) = 1.2 - (theta0^2 + theta1^2)
# by gradient ascent on the surrogate Qhat(theta|h) = 1.2 - (h0 theta0^2 + h1 theta1^2).

def toy_Q(theta):
    return 1.2 - float(theta[0] ** 2 + theta[1] ** 2)


def toy_step(member, lr):
    th = member.theta[0]
    h = member.h.astype(np.float64)
    member.theta[0] = th + lr * (-2.0 * h * th)       # ascent on Qhat
    member.t += 1


def toy_run(n_steps, lr, use_pbt, noise=None, ready_interval=4):
    """Two workers from theta = [0.9, 0.9] with h = [1, 0] and [0, 1].  With
    use_pbt the weaker copies the better every `ready_interval` iterations and
    adds noise[round] (shape (2,)) to the copied h.  Returns final Q per worker."""
    pop = [Member([np.array([0.9, 0.9])], [1.0, 0.0], index=0),
           Member([np.array([0.9, 0.9])], [0.0, 1.0], index=1)]

    def ee(pop, rnd):
        if not use_pbt:
            return None
        return exploit_explore(pop, rnd, seed=0, n_trunc=1,
                               explore_fn=lambda h, rr, r: h + np.asarray(noise[rr], dtype=np.float32))
    train(pop, n_steps, lambda m, i, s: toy_step(m, lr), lambda m, i: toy_Q(m.theta[0]),
          ready_interval, ee)
    return [toy_Q(m.theta[0]) for m in pop]
