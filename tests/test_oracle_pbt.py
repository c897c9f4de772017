"""Pins for the oracle's exploit/explore pass and training loop: brute force on
tiny populations, the invariants the paper states in prose (Section 4.1.1,
Algorithm 1) and the toy example of Figure 2."""
import itertools
import math
import os
import numpy as np
import pytest

from oracle import pbt, philox, classifier, nets

GOLD = os.path.join(os.path.dirname(__file__), "golden", "toy_figure2.txt")


def _beats(sa, a, sb, b):
    """Textbook strict order: does member a rank above member b?"""
    na, nb = math.isnan(sa), math.isnan(sb)
    if na != nb:
        return nb
    if not na and sa != sb:
        return sa > sb
    return a < b


def test_rank_bruteforce_with_ties_nan_inf():
    vals = [0.5, 0.5, -1.0, float("nan"), float("-inf"), float("inf"), 2.0, float("nan")]
    for P in range(1, 6):
        for combo in itertools.product(vals, repeat=P):
            order = pbt.rank_order(np.array(combo, dtype=np.float32))
            # rank by counting how many members beat me
            pos = [sum(_beats(combo[j], j, combo[i], i) for j in range(P) if j != i) for i in range(P)]
            assert sorted(pos) == list(range(P))
            assert [order[pos[i]] for i in range(P)] == list(range(P))


def _mk_pop(P, n_h=2, rng=None):
    rng = rng or np.random.default_rng(0)
    pop = []
    for i in range(P):
        m = pbt.Member([rng.standard_normal(5), rng.standard_normal((2, 3))],
                       rng.uniform(0.01, 1.0, size=n_h),
                       {"s0": [rng.standard_normal(5), rng.standard_normal((2, 3))]}, i)
        m.t = 10 + i
        pop.append(m)
    return pop


def _snapshot(m):
    return (b"".join(a.tobytes() for a in m.theta), b"".join(a.tobytes() for a in m.opt["s0"]),
            m.h.tobytes(), m.t, np.float32(m.p).tobytes(), m.parent)


@pytest.mark.parametrize("P", [5, 6, 7, 8])
def test_truncation_exhaustive(P):
    base = np.linspace(-1.0, 1.0, P)
    perms = list(itertools.permutations(range(P)))
    if len(perms) > 720:
        perms = perms[::len(perms) // 720]
    for n_trunc in range(0, P // 2 + 1):
        for rnd, perm in enumerate(perms):
            scores = base[list(perm)].astype(np.float32)
            pop = _mk_pop(P)
            for m, s in zip(pop, scores):
                m.p = s
            before = [_snapshot(m) for m in pop]
            anc_before = len({m.parent for m in pop})
            order, donor = pbt.exploit_explore(pop, rnd, seed=99, n_trunc=n_trunc)
            srt = sorted(range(P), key=lambda i: -scores[i])
            top, bottom = set(srt[:n_trunc]), set(srt[P - n_trunc:]) if n_trunc else set()
            assert order == srt
            for i in range(P):
                if i in bottom:
                    d = donor[i]
                    assert d in top                                   # donor from the top set
                    assert _snapshot(pop[i])[:2] == before[d][:2]      # weights + optimiser state, byte for byte
                    assert pop[i].t == pop[d].t and pop[i].parent == d
                    assert np.float32(pop[i].p) == scores[d]
                    for k in range(2):                                # exactly one of the two factors
                        lo = np.float32(np.float32(before_h(before[d])[k]) * np.float32(0.8))
                        hi = np.float32(np.float32(before_h(before[d])[k]) * np.float32(1.2))
                        assert pop[i].h[k].tobytes() in (lo.tobytes(), hi.tobytes())
                else:
                    assert donor[i] == -1
                    assert _snapshot(pop[i]) == before[i]             # untouched, hyperparameters included
            assert len({m.parent for m in pop}) <= anc_before       # ancestors can only disappear


def before_h(snap):
    return np.frombuffer(snap[2], dtype=np.float32)



def test_distinct_ancestors_never_increase():
    # Section 4.4 (lineages): copying can only remove ancestors from the population.
    P = 10
    rng = np.random.default_rng(4)
    anc = list(range(P))
    pop = _mk_pop(P)
    n_prev = P
    for rnd in range(40):
        scores = rng.standard_normal(P).astype(np.float32)
        _, donor = pbt.exploit_explore(pop, rnd, seed=5, n_trunc=2, scores=scores)
        anc = [anc[d] if d >= 0 else anc[i] for i, d in enumerate(donor)]
        assert len(set(anc)) <= n_prev
        n_prev = len(set(anc))
    assert n_prev < P


def test_donor_uniform_over_top_and_with_replacement():
    P, n_trunc = 20, 4
    scores = np.arange(P, dtype=np.float32)          # top = 19, 18, 17, 16
    hits = np.zeros(P, dtype=int)
    repeats = 0
    for rnd in range(3000):
        _, donor = pbt.truncation_select(scores, n_trunc, rnd, seed=2017)
        ds = donor[donor >= 0]
        assert len(ds) == n_trunc and set(np.nonzero(donor >= 0)[0]) == {0, 1, 2, 3}
        repeats += len(set(ds)) < n_trunc
        for d in ds:
            hits[d] += 1
    assert hits[:16].sum() == 0
    assert np.all(np.abs(hits[16:] / hits.sum() - 0.25) < 0.02)
    assert repeats > 0


def test_donor_index_formula():
    scores = np.array([3, 1, 2, 0, 5, 4], dtype=np.float32)      # order 4,5,0,2,1,3
    _, donor = pbt.truncation_select(scores, 2, 7, seed=123)
    for r in (1, 3):
        x = int(philox.philox4x32_10([7, r, philox.DOMAIN_DONOR, 0], [123, 0])[0])
        assert donor[r] == [4, 5][(x * 2) >> 32]


def test_perturb_factors_and_frequency():
    h = np.array([0.013, 0.9, 1e-5], dtype=np.float32)
    n_hi = 0
    for rnd in range(4000):
        out = pbt.perturb(h, rnd, 3, seed=11, factor_lo=0.8, factor_hi=1.2)
        for k in range(3):
            bit = int(philox.philox4x32_10([rnd, 3, philox.DOMAIN_EXPLORE, k], [11, 0])[0]) & 1
            ref = h[k] * (np.float32(1.2) if bit else np.float32(0.8))     # numpy float32 multiply
            assert out[k].tobytes() == np.float32(ref).tobytes()
            n_hi += bit
    assert abs(n_hi / 12000 - 0.5) < 0.02


def test_perturb_clamp_and_zero():
    out = pbt.perturb(np.array([0.95, 0.0], dtype=np.float32), 0, 0, seed=1, factor_lo=1.2, factor_hi=1.2,
                      h_max=[0.999, math.inf])
    assert out[0] == np.float32(0.999) and out[1] == 0.0


def test_nan_member_is_replaced():
    pop = _mk_pop(6)
    scores = np.array([0.1, np.nan, 0.3, 0.2, 0.5, 0.4], dtype=np.float32)
    pop[1].theta[0][:] = np.nan
    _, donor = pbt.exploit_explore(pop, 0, seed=3, n_trunc=1, scores=scores)
    assert donor[1] == 4 and np.isfinite(pop[1].theta[0]).all()


def test_truncation_rejects_overlap():
    with pytest.raises(ValueError):
        pbt.truncation_select(np.zeros(5, dtype=np.float32), 3, 0, 0)


def _gold():
    d = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        d[k] = float(v)
    return d


def test_toy_figure2():
    gold = _gold()
    q = pbt.toy_run(400, 0.02, use_pbt=False)
    assert abs(q[0] - gold["fixed_h_final_Q"]) < 1e-6 and abs(q[1] - gold["fixed_h_final_Q"]) < 1e-6
    assert abs(round(q[0], 1) - gold["fixed_h_paper_value"]) < 1e-12
    rng = np.random.default_rng(0)
    for trial in range(5):
        noise = rng.normal(0.0, 0.1, size=(200, 2))
        q = pbt.toy_run(800, 0.02, use_pbt=True, noise=noise)
        assert max(q) > gold["pbt_final_Q"] - 1e-2, q


def _tiny_spec(optimizer, roles):
    return classifier.ClassifierSpec([3, 5, 2], nets.ACT_RELU, optimizer, batch=4, roles=roles, seed=42)


def test_member_independence_and_random_search_limit():
    # With n_trunc = 0 PBT is random search (Section 4.1.2): each member's trajectory
    # equals a run of that member alone.
    rng = np.random.default_rng(1)
    x = rng.standard_normal((32, 3)).astype(np.float32)
    y = rng.integers(0, 2, 32).astype(np.int32)
    spec = _tiny_spec(classifier.OPT_ADAM, [classifier.ROLE_LR, classifier.ROLE_BETA1, classifier.ROLE_WD])

    def make(i):
        r = np.random.default_rng(100 + i)
        theta = [(r.standard_normal((3, 5)), r.standard_normal(5)), (r.standard_normal((5, 2)), r.standard_normal(2))]
        return classifier.new_member(spec, theta, [0.01 * (i + 1), 0.9, 1e-4], i)

    pop = [make(i) for i in range(4)]
    pbt.train(pop, 12, lambda m, i, s: classifier.step(spec, m, i, s, x, y),
              lambda m, i: classifier.evaluate(spec, m, x, y), 4,
              lambda pop, rnd: pbt.exploit_explore(pop, rnd, spec.seed, 0))
    solo = make(2)
    for s in range(12):
        classifier.step(spec, solo, 2, s, x, y)
    for a, b in zip(solo.theta, pop[2].theta):
        assert a.tobytes() == b.tobytes()
    assert pop[2].t == 12 and pop[2].parent == 2


def test_training_reduces_loss_and_batch_rows():
    rng = np.random.default_rng(2)
    means = rng.standard_normal((2, 3)) * 2
    y = rng.integers(0, 2, 256).astype(np.int32)
    x = (means[y] + rng.standard_normal((256, 3))).astype(np.float32)
    spec = _tiny_spec(classifier.OPT_SGD_MOMENTUM, [classifier.ROLE_LR])
    r = np.random.default_rng(9)
    theta = [(r.standard_normal((3, 5)) * 0.3, np.zeros(5)), (r.standard_normal((5, 2)) * 0.3, np.zeros(2))]
    m = classifier.new_member(spec, theta, [0.05], 0)
    l0 = -classifier.evaluate(spec, m, x, y)
    for s in range(200):
        classifier.step(spec, m, 0, s, x, y)
    assert -classifier.evaluate(spec, m, x, y) < 0.6 * l0
    rows = classifier.batch_rows(42, 5, 1, 4, 256)
    ref = [(int(philox.philox4x32_10([5, 1, philox.DOMAIN_BATCH, j], [42, 0])[0]) * 256) >> 32 for j in range(4)]
    assert list(rows) == ref


def test_init_hyperparameters_priors():
    # Prior ranges as in the paper's appendix tables (e.g. learning rate log-uniform, Section A.3)
    priors = [("log", 1e-4, 1e-2), ("uniform", 0.8, 0.95)]
    H = pbt.init_hyperparameters(7, 4000, priors)
    assert H.dtype == np.float32 and H.shape == (4000, 2)
    assert H[:, 0].min() >= 1e-4 * (1 - 1e-6) and H[:, 0].max() <= 1e-2 * (1 + 1e-6)
    assert H[:, 1].min() >= 0.8 and H[:, 1].max() <= 0.95
    # log-uniform: ln h is uniform, so its quartiles sit at the quarter points of [ln lo, ln hi]
    q = np.quantile(np.log(H[:, 0].astype(np.float64)), [0.25, 0.5, 0.75])
    ref = math.log(1e-4) + np.array([0.25, 0.5, 0.75]) * (math.log(1e-2) - math.log(1e-4))
    assert np.all(np.abs(q - ref) < 0.12)
    assert abs(H[:, 1].mean() - 0.875) < 0.003
    # one entry by hand from the definition
    x = int(philox.philox4x32_10([0, 5, philox.DOMAIN_INIT_H, 0], [7, 0])[0])
    u = (x + 0.5) / 2.0 ** 32
    assert H[5, 0] == np.float32(math.exp(math.log(1e-4) + u * (math.log(1e-2) - math.log(1e-4))))


def test_init_weights_distribution_and_formula():
    dims = [40, 30, 3]
    offsets = [(0, 1216), (1280, 1408)]                      # as a 64-aligned layout would place them
    layers = pbt.init_weights(11, 2, dims, offsets)
    assert [W.shape for W, _ in layers] == [(40, 30), (30, 3)] and layers[0][0].dtype == np.float32
    for (W, b), fi in zip(layers, dims[:-1]):
        bound = 1.0 / math.sqrt(fi)
        assert np.abs(W).max() < bound and np.abs(b).max() < bound
    W0 = layers[0][0].astype(np.float64)
    assert abs(W0.mean()) < 0.01 and abs(W0.var() - (1.0 / 40) / 3.0) < 0.002      # var of U(-a, a) = a^2 / 3
    # position p = 1280 + 7 is element 7 of W_1 (row 2, column 1): word 3 of counter (0, 2, INIT_W, 321)
    p = 1280 + 7
    x = int(philox.philox4x32_10([0, 2, philox.DOMAIN_INIT_W, p // 4], [11, 0])[p % 4])
    assert layers[1][0][2, 1] == np.float32((2.0 * (x + 0.5) / 2.0 ** 32 - 1.0) / math.sqrt(30))
    other = pbt.init_weights(11, 3, dims, offsets)
    assert not np.array_equal(other[0][0], layers[0][0])


# ---- binary tournament, PBT targets, resample explore (Sections 4.3.1, 4.4, 4.1.1 Explore (b)) --------

def _tiny_pop(P, rng):
    pop = []
    for i in range(P):
        m = pbt.Member([rng.standard_normal(3)], rng.uniform(0.1, 1.0, 2), {"s0": [rng.standard_normal(3)]}, i)
        m.t = 10 + i
        m.hist = [float(i)]
        pop.append(m)
    return pop


def test_binary_tournament_exhaustive_small():
    """Every member copies only from a member that ranks above it, the opponent is uniform over the
    others, and the best member never copies."""
    seen = np.zeros((6, 6), dtype=np.int64)
    for rnd in range(400):
        scores = np.array([0.3, 0.9, -1.0, 0.9, np.nan, 0.1], dtype=np.float32)
        order, donor = pbt.binary_tournament(scores, rnd, 77)
        assert order == pbt.rank_order(scores)
        place = {m: k for k, m in enumerate(order)}
        for i in range(6):
            x = philox.words(77, rnd, i, philox.DOMAIN_DONOR, 0)[0]
            j = (int(x) * 5) >> 32
            j += 1 if j >= i else 0
            assert j != i
            seen[i, j] += 1
            assert donor[i] == (j if place[j] < place[i] else -1)
        assert donor[4] != -1                                     # the NaN member loses against anyone
        assert donor[1] == -1                                     # best (tie broken by index) never copies
    off = seen[~np.eye(6, dtype=bool)]
    assert off.min() > 40 and seen.trace() == 0                   # 400 / 5 = 80 expected per pair


def test_tournament_copies_use_the_state_before_the_pass():
    """Chain 2 <- 1 <- 0: member 2 must receive member 1's OLD weights, not the ones 1 got from 0."""
    rng = np.random.default_rng(5)
    for rnd in range(300):
        pop = _tiny_pop(3, rng)
        scores = np.array([3.0, 2.0, 1.0], dtype=np.float32)
        _, donor = pbt.binary_tournament(scores, rnd, 5)
        if donor[1] == 0 and donor[2] == 1:
            old1, old0 = pop[1].theta[0].copy(), pop[0].theta[0].copy()
            old_h1 = pop[1].h.copy()
            pbt.exploit_explore(pop, rnd, 5, 0, scores=scores, mode="tournament")
            assert np.array_equal(pop[1].theta[0], old0) and np.array_equal(pop[2].theta[0], old1)
            assert pop[2].t == 11 and pop[1].t == 10 and pop[2].hist == [1.0]
            assert pop[2].h.tobytes() == pbt.perturb(old_h1, rnd, 2, 5, 0.8, 1.2).tobytes()
            return
    raise AssertionError("no chain drawn")


def test_pbt_targets_subsets():
    rng = np.random.default_rng(6)
    scores = np.array([5, 4, 3, 2, 1, 0], dtype=np.float32)
    for cw, ch in ((True, False), (False, True)):
        pop = _tiny_pop(6, rng)
        ref = [(m.theta[0].copy(), m.h.copy(), m.t, m.opt["s0"][0].copy()) for m in pop]
        _, donor = pbt.exploit_explore(pop, 0, 9, 2, scores=scores, copy_weights=cw, copy_hypers=ch)
        for r in range(6):
            d = int(donor[r])
            if d < 0:
                assert np.array_equal(pop[r].theta[0], ref[r][0]) and pop[r].h.tobytes() == ref[r][1].tobytes()
                continue
            if cw:
                assert np.array_equal(pop[r].theta[0], ref[d][0]) and pop[r].t == ref[d][2] and np.array_equal(pop[r].opt["s0"][0], ref[d][3])
                assert pop[r].p == scores[d]
            else:
                assert np.array_equal(pop[r].theta[0], ref[r][0]) and pop[r].t == ref[r][2] and pop[r].p == scores[r]
            if ch:
                assert pop[r].h.tobytes() == pbt.perturb(ref[d][1], 0, r, 9, 0.8, 1.2).tobytes()
            else:
                assert pop[r].h.tobytes() == ref[r][1].tobytes()              # neither copied nor explored


def test_resample_explore_frequency_range_and_passthrough():
    priors = [("log", 1e-4, 1e-2), ("uniform", 0.8, 0.95)]
    h = np.array([0.5, 0.5], dtype=np.float32)                                # outside both priors: a resample is visible
    hits = np.zeros(2)
    for r in range(2000):
        out = pbt.resample(h, 3, r, 11, 0.25, priors)
        for k, (kind, lo, hi) in enumerate(priors):
            if out[k] != h[k]:
                hits[k] += 1
                assert np.float32(lo) <= out[k] <= np.float32(hi)
                w = philox.words(11, 3, r, philox.DOMAIN_EXPLORE, k)
                assert int(w[1]) < 2 ** 30
                u = (int(w[2]) + 0.5) / 2.0 ** 32
                want = math.exp(math.log(lo) + u * (math.log(hi) - math.log(lo))) if kind == "log" else lo + u * (hi - lo)
                assert out[k] == np.float32(want)
    assert np.all(np.abs(hits / 2000 - 0.25) < 0.04)
    assert pbt.resample(h, 3, 0, 11, 0.0, priors).tobytes() == h.tobytes()
    always = pbt.resample(h, 3, 0, 11, 1.0, priors)
    assert always[0] != h[0] and always[1] != h[1]
    assert pbt.resample(h, 3, 0, 11, 1.0, priors, h_max=[1e-3, 0.9])[0] <= np.float32(1e-3)


# ---- t-test selection (Section 4.1.1, Exploit (a)) ---------------------------------------------------

def test_student_sf_closed_forms_and_quadrature():
    for t in (0.0, 0.3, 1.0, 2.5, 7.0):
        assert abs(pbt.student_sf(t, 1.0) - (0.5 - math.atan(t) / math.pi)) < 1e-13          # Cauchy
        assert abs(pbt.student_sf(t, 2.0) - (0.5 - t / (2.0 * math.sqrt(2.0 + t * t)))) < 1e-13
    # nu = 7.3: integrate the density numerically
    nu = 7.3
    c = math.exp(math.lgamma((nu + 1) / 2) - math.lgamma(nu / 2)) / math.sqrt(nu * math.pi)
    xs = np.linspace(1.7, 400.0, 2_000_001)
    dens = c * (1.0 + xs * xs / nu) ** (-(nu + 1) / 2)
    integral = float(((dens[:-1] + dens[1:]) * 0.5 * np.diff(xs)).sum())
    assert abs(pbt.student_sf(1.7, nu) - integral) < 1e-7
    assert abs(pbt.student_sf(3.0, 1e9) - 0.5 * math.erfc(3.0 / math.sqrt(2.0))) < 1e-9     # normal limit


def test_welch_statistic_by_hand_and_against_library():
    a, b = [1.0, 2.0, 3.0, 4.0], [2.0, 4.0, 6.0]
    t, nu, ma, mb = pbt.welch(a, b)
    # hand: var(a) = 5/3, var(b) = 4; va = 5/12, vb = 4/3; t = (4 - 2.5)/sqrt(7/4); nu = (7/4)^2 / ((5/12)^2/3 + (4/3)^2/2)
    assert (ma, mb) == (2.5, 4.0)
    assert abs(t - 1.5 / math.sqrt(1.75)) < 1e-15 and abs(nu - 1.75 ** 2 / ((5 / 12) ** 2 / 3 + (4 / 3) ** 2 / 2)) < 1e-13
    from scipy import stats
    rng = np.random.default_rng(0)
    for _ in range(20):
        x, y = rng.standard_normal(rng.integers(2, 11)), rng.standard_normal(rng.integers(2, 11)) + 0.5
        t, nu, _, _ = pbt.welch(x, y)
        ref = stats.ttest_ind(y, x, equal_var=False, alternative="greater")
        assert abs(t - ref.statistic) < 1e-12
        if t > 0:
            assert abs(pbt.student_sf(t, nu) - ref.pvalue) < 1e-12
    assert pbt.welch([1.0, 1.0], [2.0, 2.0])[0] == math.inf


def test_ttest_select_rules():
    rng = np.random.default_rng(1)
    P = 7
    hists = [list(rng.standard_normal(10) * 0.1 + m) for m in (0.0, 1.0, 0.05, 2.0, 0.0, 1.0)] + [[5.0]]   # last: one score only
    scores = np.array([np.mean(h) for h in hists], dtype=np.float32)
    n_copy = 0
    for rnd in range(200):
        order, donor = pbt.ttest_select(scores, hists, rnd, 3, 0.05)
        assert order == pbt.rank_order(scores)
        for i in range(P):
            x = philox.words(3, rnd, i, philox.DOMAIN_DONOR, 0)[0]
            j = (int(x) * (P - 1)) >> 32
            j += 1 if j >= i else 0
            if i == 6 or j == 6:
                assert donor[i] == -1                                    # too short a history on either side
                continue
            better = np.mean(hists[j]) > np.mean(hists[i])
            clear = abs(np.mean(hists[j]) - np.mean(hists[i])) > 0.5     # 0.1 noise: a gap of 1 is significant, 0.05 is not
            if better and clear:
                assert donor[i] == j
                n_copy += 1
            elif not better:
                assert donor[i] == -1
            elif {i, j} == {0, 2} or {i, j} == {2, 4} or {i, j} == {0, 4} or {i, j} == {1, 5}:
                assert donor[i] == -1 or pbt.student_sf(*pbt.welch(hists[i], hists[j])[:2]) < 0.05
    assert n_copy > 100
    # alpha = 1 turns the test into "higher mean wins"; alpha = 0 never copies
    _, d1 = pbt.ttest_select(scores, hists, 0, 3, 1.0)
    _, d0 = pbt.ttest_select(scores, hists, 0, 3, 0.0)
    assert np.all(d0 == -1) and (d1 >= 0).sum() >= (pbt.ttest_select(scores, hists, 0, 3, 0.05)[1] >= 0).sum()


def test_init_segments_matches_init_weights_and_constants():
    dims, offsets = [5, 7, 3], [(0, 64), (128, 192)]
    layers = pbt.init_weights(11, 2, dims, offsets)
    segs = pbt.init_segments(11, 2, [(0, (5, 7), 5, 0.0), (64, (7,), 5, 0.0), (128, (7, 3), 7, 0.0), (192, (3,), 7, 0.0), (256, (4,), 0, 1.0)])
    for (W, b), k in zip(layers, (0, 2)):
        assert W.tobytes() == segs[k].tobytes() and b.tobytes() == segs[k + 1].tobytes()
    assert np.all(segs[4] == 1.0)
    assert np.all(np.abs(segs[0]) < 1 / math.sqrt(5)) and abs(float(segs[2].mean())) < 0.2
