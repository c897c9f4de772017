"""The actor-critic workload on the GPU against the oracle: A2C loss and update with RMSProp, the
return history behind the score, and exploit/explore carrying the history along."""
import numpy as np
import pytest

from paper_1711_09846_amd import binding, workloads
from tests.harness import A2CPair

pytestmark = pytest.mark.gpu

TOL_BF16 = 1e-2
FLOOR = 1e-2    # |gpu - ref| / max(|ref|, FLOOR); the loss mixes O(1) log-probabilities, squared value errors and entropies


def _reduced(P=6):
    return workloads.A2C_MLP.replace(P=P, dims=[24, 72, 40, 19], batch=5, unroll=6, n_train=50, n_trunc=1, latent=4,
                                     priors=[("log", 1e-4, 2e-3), ("log", 1e-4, 1e-2)])


def _hist_equal(pair, members):
    got = pair.gpu.history()
    for i in members:
        ref = [float(v) for v in pair.ref[i].hist]
        assert len(got[i]) == len(ref) and np.allclose(got[i], ref, rtol=2e-7, atol=1e-7), (i, got[i], ref)


def test_a2c_reduced_free_running_window():
    pair = A2CPair(_reduced())
    g, P = pair.gpu, pair.wl.P
    assert np.all(np.isneginf(_eval(g)))                              # no unroll yet
    worst = dict(w=0.0, s0=0.0, loss=0.0, score=0.0)
    rnd = 0
    for s in range(26):
        g.step(pair.d_pool, s)
        loss_ref = pair.step_ref(s)
        loss = g.get(binding.ARR_LOSS)
        worst["loss"] = max(worst["loss"], float(np.max(np.abs(loss - loss_ref) / np.maximum(np.abs(loss_ref), FLOOR))))
        for i in range(P):
            worst["w"] = max(worst["w"], pair.member_errors(i, binding.ARR_W32, "theta")[0])
            worst["s0"] = max(worst["s0"], pair.member_errors(i, binding.ARR_OPT0, "s0")[1])
        assert worst["w"] <= TOL_BF16 and worst["loss"] <= TOL_BF16, (s, worst)
        _hist_equal(pair, range(P))
        if (s + 1) % 4 == 0:
            sc = _eval(g)
            sc_ref = pair.eval_ref()
            worst["score"] = max(worst["score"], float(np.max(np.abs(sc - sc_ref) / np.maximum(np.abs(sc_ref), FLOOR))))
            assert worst["score"] <= 1e-6
            g.exploit_explore(rnd)
            order, donor = pair.exploit_ref(rnd, sc)
            assert list(g.get(binding.ARR_ORDER)) == order and np.array_equal(g.get(binding.ARR_DONOR), donor)
            assert g.get(binding.ARR_HYPER).tobytes() == np.stack([pair.ref[i].h for i in range(P)]).tobytes()
            _hist_equal(pair, range(P))                               # the history travelled with the weights
            rnd += 1
    print("a2c reduced:", {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)


def _eval(g):
    g.eval()
    return g.get(binding.ARR_SCORE)


def test_a2c_full_size_steps_score_and_copy():
    """P = 128, torso 512-256-256, head 18 + 1, 32 trajectories x 20 transitions (672 rows per member).
    Four sampled members are followed by the oracle, re-synchronised before every step."""
    from oracle import pbt as opbt
    wl = workloads.A2C_MLP
    H0 = workloads.initial_hypers(wl, 6)
    sample = sorted({int(np.argmax(H0[:, 0])), int(np.argmax(H0[:, 1])), 3, 77})
    pair = A2CPair(wl, ref_members=sample)
    g = pair.gpu
    worst = dict(step=0.0, s0=0.0, loss=0.0, score=0.0)
    for s in range(12):
        for i in sample:
            pair.sync_ref_from_gpu(i)
        g.step(pair.d_pool, s)
        loss_ref = pair.step_ref(s)
        loss = g.get(binding.ARR_LOSS)[sample]
        worst["loss"] = max(worst["loss"], float(np.max(np.abs(loss - loss_ref) / np.maximum(np.abs(loss_ref), FLOOR))))
        for i in sample:
            worst["step"] = max(worst["step"], pair.member_errors(i, binding.ARR_W32, "theta")[0])
            worst["s0"] = max(worst["s0"], pair.member_errors(i, binding.ARR_OPT0, "s0")[1])
        assert worst["step"] <= TOL_BF16 and worst["loss"] <= TOL_BF16, (s, worst)
        _hist_equal(pair, sample)
    sc = _eval(g)
    worst["score"] = float(np.max(np.abs(sc[sample] - pair.eval_ref())))
    assert worst["score"] <= 1e-6
    before = {w: g.get(w) for w in (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_W16, binding.ARR_HIST, binding.ARR_HYPER)}
    g.exploit_explore(0)
    order, donor = opbt.truncation_select(sc, wl.n_trunc, 0, pair.seed)
    assert list(g.get(binding.ARR_ORDER)) == order and np.array_equal(g.get(binding.ARR_DONOR), donor)
    assert (donor >= 0).sum() == 25
    after = {w: g.get(w) for w in before}
    for r in range(wl.P):
        src = donor[r] if donor[r] >= 0 else r
        for w in (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_W16, binding.ARR_HIST):
            assert after[w][r].tobytes() == before[w][src].tobytes()
        href = before[binding.ARR_HYPER][r] if donor[r] < 0 else opbt.perturb(
            before[binding.ARR_HYPER][src], 0, r, pair.seed, wl.perturb[0], wl.perturb[1], wl.h_max)
        assert after[binding.ARR_HYPER][r].tobytes() == href.tobytes()
    print("a2c full size:", {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)


@pytest.mark.parametrize("alpha", [0.05, 0.5, 1.0])
def test_a2c_ttest_selection_bit_exact(alpha):
    """Section 4.1.1 Exploit (a): opponent drawn uniformly, Welch's test on the last 10 unroll returns.
    Both sides decide from the same float32 histories in double precision."""
    wl = _reduced(P=12).replace(exploit_mode=2, ttest_alpha=alpha)
    pair = A2CPair(wl)
    g, P = pair.gpu, wl.P
    n_copy = n_chain = 0
    rnd = 0
    for s in range(16):
        g.step(pair.d_pool, s)
        if s == 0:                                                    # one entry only: nobody may copy
            g.exploit_explore(99)
            assert np.all(g.get(binding.ARR_DONOR) == -1)
        if s >= 3 and s % 4 == 3:
            for i in range(P):
                pair.sync_ref_from_gpu(i)
            sc = _eval(g)
            before = {w: g.get(w).copy() for w in (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_W16, binding.ARR_HIST, binding.ARR_HYPER)}
            g.exploit_explore(rnd)
            order, donor = pair.exploit_ref(rnd, sc)
            assert list(g.get(binding.ARR_ORDER)) == order and np.array_equal(g.get(binding.ARR_DONOR), donor), (s, donor)
            n_copy += int((donor >= 0).sum())
            n_chain += sum(1 for i in range(P) if donor[i] >= 0 and donor[donor[i]] >= 0)
            after = {w: g.get(w) for w in before}
            for i in range(P):
                src = donor[i] if donor[i] >= 0 else i
                for w in (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_W16, binding.ARR_HIST):
                    assert after[w][i].tobytes() == before[w][src].tobytes()
            assert after[binding.ARR_HYPER].tobytes() == np.stack([pair.ref[i].h for i in range(P)]).tobytes()
            _hist_equal(pair, range(P))
            rnd += 1
    assert n_copy > 0
    print("t-test selection alpha %.2f: %d copies, %d of them from a member that was itself overwritten" % (alpha, n_copy, n_chain), flush=True)


def _one_kernel_unroll_shape():
    """A shape the single-kernel unroll covers (at most 32 trajectories, hidden widths 64 / 128 / 256, observation
    width a multiple of 64), with fewer than 32 trajectories, an odd latent size and two different hidden widths."""
    return workloads.A2C_MLP.replace(P=4, dims=[64, 128, 64, 7], n_actions=6, batch=20, unroll=5, n_train=50, n_trunc=1, latent=5,
                                     priors=[("log", 1e-4, 2e-3), ("log", 1e-4, 1e-2)])


@pytest.mark.parametrize("shape", ["kernel_per_round", "one_kernel"])
def test_a2c_on_policy_unrolls_against_the_oracle(shape):
    """Section 4.1.1: agents act with their current policy.  Every step the GPU generates the unroll; the oracle
    (a) replays the latent system along the GPU's actions and must reproduce observations and rewards, (b) makes
    its own choice at every transition from its own logits: it may differ from the GPU's only where the uniform
    draw lies within 1e-3 of an edge of the cdf (float32 against float64 logits), and on fewer than 1 % of the
    choices, (c) takes its step on the GPU's unroll and must stay within the bf16 tolerance, free-running."""
    from oracle import nets
    wl = (_reduced() if shape == "kernel_per_round" else _one_kernel_unroll_shape()).replace(on_policy=1)
    pair = A2CPair(wl)
    g, P = pair.gpu, wl.P
    n_choices = n_differ = n_obs = n_obs_differ = 0
    worst = dict(w=0.0, loss=0.0, reward=0.0, score=0.0)
    rnd = 0
    for s in range(16):
        before = {i: pair.oa.params_of(pair.ref[i]) for i in range(P)}
        before = {i: [(W.copy(), b.copy()) for W, b in before[i]] for i in range(P)}
        g.step(pair.d_pool, s)
        for i in range(P):
            obs_g, act_g, rew_g = pair.gpu_unroll(i)
            assert act_g.min() >= 0 and act_g.max() < wl.n_actions
            obs_o, act_o, rew_o, margin = pair.env_mod.rollout(pair.spec, pair.env, before[i], i, s, forced_actions=act_g)
            differ = act_o != act_g
            assert np.all(margin[differ] < 1e-3), (s, i, margin[differ])
            n_choices += act_g.size
            n_differ += int(differ.sum())
            obs_o16 = nets.round_bf16(obs_o.astype(np.float64))
            off = obs_o16 != obs_g
            # one bf16 step at most (the device draws the observation noise to float accuracy, about 2e-7 of a value
            # of order one: next to zero, where bf16 is finer than that, the absolute distance is what is bounded)
            assert np.all(np.abs(obs_o16 - obs_g)[off] <= np.maximum(2.0 ** -7 * np.abs(obs_g)[off], 2e-6)), (s, i)
            n_obs += obs_g.size
            n_obs_differ += int(off.sum())
            worst["reward"] = max(worst["reward"], float(np.max(np.abs(rew_o.astype(np.float64) - rew_g))))
        loss_ref = pair.step_ref(s)
        loss = g.get(binding.ARR_LOSS)
        worst["loss"] = max(worst["loss"], float(np.max(np.abs(loss - loss_ref) / np.maximum(np.abs(loss_ref), FLOOR))))
        for i in range(P):
            worst["w"] = max(worst["w"], pair.member_errors(i, binding.ARR_W32, "theta")[0])
        assert worst["w"] <= TOL_BF16 and worst["loss"] <= TOL_BF16 and worst["reward"] <= 1e-5, (s, worst)
        _hist_equal(pair, range(P))
        if (s + 1) % 4 == 0:
            sc = _eval(g)
            worst["score"] = max(worst["score"], float(np.max(np.abs(sc - pair.eval_ref()))))
            assert worst["score"] <= 1e-5 and len(set(sc.tolist())) == P       # every member earned its own score
            g.exploit_explore(rnd)
            order, donor = pair.exploit_ref(rnd, sc)
            assert list(g.get(binding.ARR_ORDER)) == order and np.array_equal(g.get(binding.ARR_DONOR), donor)
            assert g.get(binding.ARR_HYPER).tobytes() == np.stack([pair.ref[i].h for i in range(P)]).tobytes()
            rnd += 1
    assert n_differ <= 0.01 * n_choices and n_obs_differ <= 1e-3 * n_obs, (n_differ, n_choices, n_obs_differ, n_obs)
    print("a2c on-policy: %d of %d choices differ (all next to a cdf edge), %d of %d observations round the other way;"
          % (n_differ, n_choices, n_obs_differ, n_obs), {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)


def test_a2c_on_policy_full_size_steps():
    """P = 128 at the full shape, a few on-policy steps: sampled members' unrolls replayed by the oracle, their
    steps within the tolerance, and scores that differ between members."""
    from oracle import nets
    wl = workloads.A2C_MLP_ON_POLICY
    sample = [3, 40, 77, 120]
    pair = A2CPair(wl, ref_members=sample)
    g = pair.gpu
    worst = dict(w=0.0, loss=0.0, reward=0.0)
    n_choices = n_differ = 0
    for s in range(5):
        before = {i: [(W.copy(), b.copy()) for W, b in pair.oa.params_of(pair.ref[i])] for i in sample}
        g.step(pair.d_pool, s)
        for i in sample:
            obs_g, act_g, rew_g = pair.gpu_unroll(i)
            obs_o, act_o, rew_o, margin = pair.env_mod.rollout(pair.spec, pair.env, before[i], i, s, forced_actions=act_g)
            differ = act_o != act_g
            assert np.all(margin[differ] < 1e-3)
            n_choices += act_g.size
            n_differ += int(differ.sum())
            assert np.mean(nets.round_bf16(obs_o.astype(np.float64)) != obs_g) <= 1e-3
            worst["reward"] = max(worst["reward"], float(np.max(np.abs(rew_o.astype(np.float64) - rew_g))))
        loss_ref = pair.step_ref(s)
        loss = g.get(binding.ARR_LOSS)[sample]
        worst["loss"] = max(worst["loss"], float(np.max(np.abs(loss - loss_ref) / np.maximum(np.abs(loss_ref), FLOOR))))
        for i in sample:
            worst["w"] = max(worst["w"], pair.member_errors(i, binding.ARR_W32, "theta")[0])
        assert worst["w"] <= TOL_BF16 and worst["loss"] <= TOL_BF16 and worst["reward"] <= 1e-5, (s, worst)
        _hist_equal(pair, sample)
    sc = _eval(g)
    assert len(set(sc.tolist())) > 100 and n_differ <= 0.01 * n_choices
    print("a2c on-policy full size:", {k: float("%.3g" % v) for k, v in worst.items()}, "choices differing:", n_differ, "of", n_choices, flush=True)
