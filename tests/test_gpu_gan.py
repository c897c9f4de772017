"""The GAN workload on the GPU against the oracle: discriminator and generator updates, losses,
the MMD score, and exploit/explore copying both networks."""
import numpy as np
import pytest

from paper_1711_09846_amd import binding, workloads
from tests.harness import GanPair

pytestmark = pytest.mark.gpu

TOL_BF16 = 1e-2
FLOOR = 1.0     # losses are softplus of O(1) logits, the score a difference of kernel means of order 1


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
