"""The GAN workload on the GPU against the oracle: discriminator and generator updates, losses,
the MMD score, and exploit/explore copying both networks."""
import numpy as np
import pytest

from paper_1711_09846_amd import binding, workloads
from tests.harness import GanPair

pytestmark = pytest.mark.gpu

TOL_BF16 = 1e-2
FLOOR = 1e-2    # |gpu - ref| / max(|ref|, FLOOR) for losses (softplus of O(1) logits) and scores (kernel means, 1e-2 .. 0.5)

# WGAN-GP losses: a difference of critic means plus 10 x a mean squared deviation of gradient norms from 1; their
# absolute error is set by those O(1) terms and does not shrink when the terms cancel
FLOOR_WGAN = 1.0


def _reduced(P=5):
    # several MFMA tiles with ragged tails in every dimension; 200 eval rows = 1.6 tiles
    return workloads.GAN_MLP.replace(P=P, dims=[16, 72, 40], dims2=[40, 136, 24, 1], batch=24, n_train=1024, n_eval=200,
                                     n_trunc=1, priors=[("log", 1e-4, 2e-3), ("log", 1e-4, 2e-3)], n_modes=4, rank=8)


def test_gan_reduced_free_running_window():
    pair = GanPair(_reduced())
    g = pair.gpu
    worst = dict(w=0.0, loss=0.0, score=0.0, m=0.0)
    rnd = 0
    for s in range(18):
        g.step(pair.d_train, s)
        loss_ref = pair.step_ref(s)
        loss = g.get(binding.ARR_LOSS)
        worst["loss"] = max(worst["loss"], float(np.max(np.abs(loss - loss_ref) / np.maximum(np.abs(loss_ref), FLOOR))))
        for i in range(pair.wl.P):
            worst["w"] = max(worst["w"], pair.member_errors(i, binding.ARR_W32, "theta")[0])
            worst["m"] = max(worst["m"], pair.member_errors(i, binding.ARR_OPT0, "s0")[1])
        assert worst["w"] <= TOL_BF16 and worst["loss"] <= TOL_BF16, (s, worst)
        if (s + 1) % 6 == 0:
            g.eval(pair.d_eval)
            sc = g.get(binding.ARR_SCORE)
            sc_ref = pair.eval_ref()
            worst["score"] = max(worst["score"], float(np.max(np.abs(sc - sc_ref) / np.maximum(np.abs(sc_ref), FLOOR))))
            assert worst["score"] <= TOL_BF16, (s, sc, sc_ref)
            assert np.all(sc <= 1e-6)                                  # MMD^2 >= 0 up to rounding
            g.exploit_explore(rnd)
            order, donor = pair.exploit_ref(rnd, sc)
            assert list(g.get(binding.ARR_ORDER)) == order and np.array_equal(g.get(binding.ARR_DONOR), donor)
            assert g.get(binding.ARR_HYPER).tobytes() == np.stack([pair.ref[i].h for i in range(pair.wl.P)]).tobytes()
            rnd += 1
    print("gan reduced:", {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)


def test_gan_one_network_frozen_by_zero_learning_rate():
    wl = _reduced(P=2)
    pair = GanPair(wl)
    H = np.array([[0.0, 1e-3], [1e-3, 0.0]], dtype=np.float32)
    pair.gpu.set(binding.ARR_HYPER, H)
    before = pair.gpu.get(binding.ARR_W32).copy()
    pair.gpu.step(pair.d_train, 0)
    after = pair.gpu.get(binding.ARR_W32)
    cut = pair.gpu.layout.w_off[len(wl.dims) - 1]                      # first discriminator element
    assert np.array_equal(after[0, :cut], before[0, :cut]) and not np.array_equal(after[0, cut:], before[0, cut:])
    assert np.array_equal(after[1, cut:], before[1, cut:]) and not np.array_equal(after[1, :cut], before[1, :cut])


def test_gan_full_size_steps_and_score():
    """P = 32, G 128-512-512-784, D 784-512-512-1, batch 64, 2048-row MMD score.  All members on the GPU;
    four sampled members followed by the oracle, re-synchronised before every step (bound on what
    one step adds), then the score and an exploit/explore round checked byte for byte."""
    from oracle import pbt as opbt
    wl = workloads.GAN_MLP
    H0 = workloads.initial_hypers(wl, 6)
    sample = sorted({int(np.argmax(H0[:, 0])), int(np.argmin(H0[:, 1])), 7, 20})
    pair = GanPair(wl, ref_members=sample)
    g = pair.gpu
    worst = dict(step=0.0, loss=0.0, score=0.0)
    for s in range(12):
        for i in sample:
            pair.sync_ref_from_gpu(i)
        g.step(pair.d_train, s)
        loss_ref = pair.step_ref(s)
        loss = g.get(binding.ARR_LOSS)[sample]
        worst["loss"] = max(worst["loss"], float(np.max(np.abs(loss - loss_ref) / np.maximum(np.abs(loss_ref), FLOOR))))
        for i in sample:
            worst["step"] = max(worst["step"], pair.member_errors(i, binding.ARR_W32, "theta")[0])
            assert int(g.get(binding.ARR_T, i)[0]) == pair.ref[i].t
        assert worst["step"] <= TOL_BF16 and worst["loss"] <= TOL_BF16, (s, worst)
    for i in sample:
        pair.sync_ref_from_gpu(i)
    g.eval(pair.d_eval)
    sc = g.get(binding.ARR_SCORE)
    sc_ref = pair.eval_ref()
    worst["score"] = float(np.max(np.abs(sc[sample] - sc_ref) / np.maximum(np.abs(sc_ref), FLOOR)))
    assert worst["score"] <= TOL_BF16, (sc[sample], sc_ref)
    before = {w: g.get(w) for w in (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_OPT1, binding.ARR_W16, binding.ARR_HYPER)}
    g.exploit_explore(0)
    order, donor = opbt.truncation_select(sc, wl.n_trunc, 0, pair.seed)
    assert list(g.get(binding.ARR_ORDER)) == order and np.array_equal(g.get(binding.ARR_DONOR), donor)
    after = {w: g.get(w) for w in before}
    for r in range(wl.P):
        src = donor[r] if donor[r] >= 0 else r
        for w in (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_OPT1, binding.ARR_W16):
            assert after[w][r].tobytes() == before[w][src].tobytes()             # generator AND discriminator travel
        href = before[binding.ARR_HYPER][r] if donor[r] < 0 else opbt.perturb(
            before[binding.ARR_HYPER][src], 0, r, pair.seed, wl.perturb[0], wl.perturb[1], wl.h_max)
        assert after[binding.ARR_HYPER][r].tobytes() == href.tobytes()
    print("gan full size:", {k: float("%.3g" % v) for k, v in worst.items()}, "scores", sc[sample], sc_ref, flush=True)


def test_wgan_gp_reduced_free_running_window():
    """Section 4.3.1: K critic updates on the WGAN-GP objective, then one generator update, per step."""
    wl = _reduced(P=4).replace(objective="wgan_gp", n_critic=3, gp_weight=10.0, perturb=(0.5, 2.0))
    pair = GanPair(wl)
    g = pair.gpu
    worst = dict(w=0.0, loss=0.0, score=0.0, m=0.0)
    rnd = 0
    for s in range(12):
        g.step(pair.d_train, s)
        loss_ref = pair.step_ref(s)
        loss = g.get(binding.ARR_LOSS)
        worst["loss"] = max(worst["loss"], float(np.max(np.abs(loss - loss_ref) / np.maximum(np.abs(loss_ref), FLOOR_WGAN))))
        for i in range(pair.wl.P):
            worst["w"] = max(worst["w"], pair.member_errors(i, binding.ARR_W32, "theta")[0])
            worst["m"] = max(worst["m"], pair.member_errors(i, binding.ARR_OPT0, "s0")[1])
            assert int(g.get(binding.ARR_T, i)[0]) == pair.ref[i].t == s + 1
        assert worst["w"] <= TOL_BF16 and worst["loss"] <= TOL_BF16, (s, worst, loss, loss_ref)
        if (s + 1) % 4 == 0:
            g.eval(pair.d_eval)
            sc = g.get(binding.ARR_SCORE)
            sc_ref = pair.eval_ref()
            worst["score"] = max(worst["score"], float(np.max(np.abs(sc - sc_ref) / np.maximum(np.abs(sc_ref), FLOOR))))
            assert worst["score"] <= TOL_BF16, (s, sc, sc_ref)
            g.exploit_explore(rnd)
            order, donor = pair.exploit_ref(rnd, sc)
            assert list(g.get(binding.ARR_ORDER)) == order and np.array_equal(g.get(binding.ARR_DONOR), donor)
            Hg = g.get(binding.ARR_HYPER)
            assert Hg.tobytes() == np.stack([pair.ref[i].h for i in range(pair.wl.P)]).tobytes()
            rnd += 1
    print("wgan-gp reduced:", {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)


def test_wgan_gp_one_critic_step_gradient_against_the_oracle():
    """One step with a single critic update and zero learning rates: the gradient buffer holds the critic's
    gradient (Wasserstein terms + penalty) and then the generator's, compared array by array."""
    from oracle import gan as og
    wl = _reduced(P=3).replace(objective="wgan_gp", n_critic=1, gp_weight=10.0)
    pair = GanPair(wl)
    g = pair.gpu
    g.set(binding.ARR_HYPER, np.zeros((3, 2), dtype=np.float32))
    g.step(pair.d_train, 0)
    G = g.get(binding.ARR_GRAD).astype(np.float64)
    lay, shapes = g.layout, g.layer_shapes
    n_g = pair.spec.n_g
    for i in range(3):
        m = pair.ref[i]
        rows = og.philox.bounded(og.philox.words(pair.seed, 0, i, og.philox.DOMAIN_BATCH, np.arange(wl.batch))[..., 0], len(pair.train_x))
        _, gd = og.critic_loss_and_grads(pair.spec, m, pair.train_x[rows], og.latents(pair.seed, 0, i, 3, wl.batch, wl.dims[0]),
                                         og.gp_eps(pair.seed, 0, i, 0, wl.batch))
        _, gg = og.wgan_generator_loss_and_grads(pair.spec, m, og.latents(pair.seed, 0, i, 1, wl.batch, wl.dims[0]))
        for l, (gW, gb) in enumerate(list(gg) + list(gd)):
            fi, fo = shapes[l]
            got_w = G[i, lay.w_off[l]:lay.w_off[l] + fi * fo].reshape(fi, fo)
            got_b = G[i, lay.b_off[l]:lay.b_off[l] + fo]
            assert np.linalg.norm(got_w - gW) <= TOL_BF16 * np.linalg.norm(gW), (i, l, "W")
            assert np.linalg.norm(got_b - gb) <= TOL_BF16 * max(np.linalg.norm(gb), 1e-3), (i, l, "b")


def test_wgan_gp_full_size_steps():
    """P = 32 at the full shape with 5 critic updates per step: sampled members per step against the oracle."""
    wl = workloads.GAN_MLP_WGAN_GP
    sample = [2, 13, 21, 30]
    pair = GanPair(wl, ref_members=sample)
    g = pair.gpu
    worst = dict(step=0.0, loss=0.0)
    for s in range(6):
        for i in sample:
            pair.sync_ref_from_gpu(i)
        g.step(pair.d_train, s)
        loss_ref = pair.step_ref(s)
        loss = g.get(binding.ARR_LOSS)[sample]
        worst["loss"] = max(worst["loss"], float(np.max(np.abs(loss - loss_ref) / np.maximum(np.abs(loss_ref), FLOOR_WGAN))))
        for i in sample:
            worst["step"] = max(worst["step"], pair.member_errors(i, binding.ARR_W32, "theta")[0])
        assert worst["step"] <= TOL_BF16 and worst["loss"] <= TOL_BF16, (s, worst, loss, loss_ref)
    print("wgan-gp full size:", {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)
