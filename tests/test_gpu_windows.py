"""100-step windows of the bf16 workloads at their full shapes: the whole population runs on the GPU, a
sample of members is followed by the oracle in three ways at once.

  per step      an oracle twin takes over the GPU's state before every step (weights, optimiser state,
                update count, hyperparameters): loss, updated weights and optimiser state of that one step
                must agree within the bf16 tolerance, at every step of the window;
  free-running  a second twin never looks at the GPU again after the common start (except that a member
                overwritten by exploit restarts from the copy it received): its distance from the GPU is the
                accumulated drift;
  conditioning  a third twin runs free from a starting point moved by 1e-4 (relative, random signs): its
                distance from the second twin is what the trajectory itself does to a difference of the
                size of one step's rounding.  Members whose learning rate makes training unstable amplify
                such a difference without bound; no two implementations stay together there.

The free-running drift is asserted against the tolerance wherever the trajectory is well conditioned
(conditioning twin within COND_OK of the free twin) and reported everywhere.  At chosen steps a fourth,
plain float64 twin (no bf16 rounding model at all) takes one step from the GPU's state: the distance of the
GPU from exact arithmetic.  The loss is asserted against the tolerance.  For the weights the comparison
splits by the sign of the update: Adam's (and RMSProp's) early updates are lr * sign(g) whatever |g| is, so
where bf16 rounding flips the sign of a near-zero gradient element the two updates differ by 2 lr, a
property of the update rule (with lr = 1e-2 and weights of rms 0.04, a share of 0.1 % of flipped elements
already moves the weight vector by 2 %); the weights are asserted on the elements whose update has the same
sign on both sides, and the share of the others and the distance over all elements are reported.
Scores are compared at the exploit points, and the exploit/explore pass is checked byte for byte."""
import copy
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
from threadpoolctl import threadpool_limits

from oracle import pbt as opbt
from paper_1711_09846_amd import binding, workloads
from tests import harness as hs

pytestmark = pytest.mark.gpu

TOL = 1e-2          # bf16 compute, relative
LOSS_FLOOR = 1e-2   # |gpu - ref| / max(|ref|, LOSS_FLOOR) for losses and scores
BIAS_FLOOR = 1e-2   # biases start at (or near) zero: compared at no smaller scale than an rms of 1e-2
COND_OK = 1e-3      # a 1e-4 difference has grown by less than 10x: the trajectory is well conditioned
_pool = ThreadPoolExecutor(8)


def _rel(a, b, floor=LOSS_FLOOR):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return float(np.max(np.abs(a - b) / np.maximum(np.abs(b), floor)))


def _moved(m, rng, eps=1e-4):
    out = copy.deepcopy(m)
    out.theta = [a * (1.0 + eps * rng.choice([-1.0, 1.0], size=a.shape)) for a in out.theta]
    return out


def _flat(pair, arrays):
    """One vector of all parameters (the transformer's key biases, on which the network does not depend, left out)."""
    d = pair.wl.d_model if isinstance(pair, hs.TransformerPair) else 0
    names = [n for n, _ in pair.spec.param_shapes()] if d else [""] * len(arrays)
    return np.concatenate([np.delete(a, np.s_[d:2 * d]) if n.startswith("bqkv") else np.ravel(a) for n, a in zip(names, arrays)])


def _state_arrays(pair, m):
    out = [("theta", binding.ARR_W32, m.theta)]
    if "s0" in m.opt:
        out.append(("s0", binding.ARR_OPT0, m.opt["s0"]))
    if "s1" in m.opt:
        out.append(("s1", binding.ARR_OPT1, m.opt["s1"]))
    return out


def run_window(pair, sample, n_steps, exploit_after, exact_at=(0, 9, 49, 99), with_conditioning=True, per_array=True, label=""):
    g, wl = pair.gpu, pair.wl
    t_start = time.time()
    rng = np.random.default_rng(11)
    free = {i: pair.ref[i] for i in sample}
    forced = {i: copy.deepcopy(pair.ref[i]) for i in sample}
    near = {i: _moved(pair.ref[i], rng) for i in sample} if with_conditioning else {}
    xspec = hs.exact_spec(pair)
    worst = dict(step_loss=0.0, step_w=0.0, step_w_array=0.0, step_state=0.0, score=0.0, exact_loss=0.0, exact_w=0.0,
                 exact_w_same_sign=0.0, exact_sign_flips=0.0)
    drift = {i: [] for i in sample}      # free-running distance per step
    cond = {i: [] for i in sample}       # conditioning-twin distance per step
    n_asserted = 0
    rnd = 0
    for s in range(n_steps):
        for i in sample:
            hs.sync_member(pair, forced[i], i)
        exact = {i: copy.deepcopy(forced[i]) for i in sample} if s in exact_at else {}
        before = {i: [a.copy() for a in forced[i].theta] for i in exact}
        g.step(hs.train_inputs(pair), s)
        loss_gpu = g.get(binding.ARR_LOSS).reshape(wl.P, -1)
        jobs = [(forced, i, None) for i in sample] + [(free, i, None) for i in sample] + [(near, i, None) for i in near] + \
               [(exact, i, xspec) for i in exact]
        with threadpool_limits(limits=2):       # 8 oracle members at a time, two BLAS threads each
            losses = list(_pool.map(lambda j: hs.oracle_step(pair, j[0][j[1]], j[1], s, j[2]), jobs))
        for (who, i, _), loss in zip(jobs, losses):
            if who is forced:
                worst["step_loss"] = max(worst["step_loss"], _rel(loss_gpu[i], loss))
                for what, which, arrs in _state_arrays(pair, forced[i]):
                    per, whole = hs.array_distances(pair, hs.gpu_arrays(pair, i, which), arrs, bias_floor=BIAS_FLOOR)
                    if what == "theta":
                        worst["step_w"], worst["step_w_array"] = max(worst["step_w"], whole), max(worst["step_w_array"], per.max())
                    else:
                        worst["step_state"] = max(worst["step_state"], whole)
                assert int(g.get(binding.ARR_T, i)[0]) == forced[i].t
            elif who is exact:
                worst["exact_loss"] = max(worst["exact_loss"], _rel(loss_gpu[i], loss))
                w_gpu, w_exact, w_before = (_flat(pair, a) for a in (hs.gpu_arrays(pair, i, binding.ARR_W32), exact[i].theta, before[i]))
                same = np.sign(w_gpu - w_before) == np.sign(w_exact - w_before)
                worst["exact_w"] = max(worst["exact_w"], np.linalg.norm(w_gpu - w_exact) / np.linalg.norm(w_exact))
                worst["exact_w_same_sign"] = max(worst["exact_w_same_sign"], np.linalg.norm((w_gpu - w_exact)[same]) / np.linalg.norm(w_exact[same]))
                moved = (w_exact != w_before) | (w_gpu != w_before)
                worst["exact_sign_flips"] = max(worst["exact_sign_flips"], float(np.mean(~same[moved])) if moved.any() else 0.0)
        # every step of the window: what one step adds, against the bf16 oracle and (sampled) against exact arithmetic
        assert worst["step_loss"] <= TOL and worst["step_w"] <= TOL and (worst["step_w_array"] <= TOL or not per_array), (label, s, worst)
        assert worst["exact_loss"] <= TOL and worst["exact_w_same_sign"] <= TOL, (label, s, worst)
        for i in sample:
            w_gpu = hs.gpu_arrays(pair, i, binding.ARR_W32)
            drift[i].append(hs.array_distances(pair, w_gpu, free[i].theta, bias_floor=BIAS_FLOOR)[1])
            if near:
                cond[i].append(hs.array_distances(pair, near[i].theta, free[i].theta, bias_floor=BIAS_FLOOR)[1])
                if cond[i][-1] <= COND_OK:
                    n_asserted += 1
                    assert drift[i][-1] <= TOL, (label, "free-running drift of a well-conditioned member", s, i, drift[i][-1], cond[i][-1])
                # everywhere: the GPU stays within an order of magnitude of what the trajectory does to a 1e-4 difference
                assert drift[i][-1] <= max(TOL, 10.0 * cond[i][-1]), (label, "drift beyond what the trajectory does to a 1e-4 difference", s, i, drift[i][-1], cond[i][-1])
        if s + 1 in exploit_after:
            g.eval(hs.eval_inputs(pair))
            sc = g.get(binding.ARR_SCORE)
            for i in sample:
                hs.sync_member(pair, forced[i], i)
            sc_ref = list(_pool.map(lambda i: hs.oracle_eval(pair, forced[i], i), sample))
            worst["score"] = max(worst["score"], _rel(sc[sample], sc_ref))
            assert worst["score"] <= TOL, (label, s, sc[sample], sc_ref)
            arrays = [binding.ARR_W32, binding.ARR_OPT0, binding.ARR_W16, binding.ARR_HYPER, binding.ARR_T]
            arrays += [binding.ARR_OPT1] if wl.optimizer == workloads.OPT_ADAM else []
            arrays += [binding.ARR_HIST] if wl.kind == workloads.WL_A2C else []
            before = {w: g.get(w) for w in arrays}
            g.exploit_explore(rnd)
            order, donor = opbt.truncation_select(sc, wl.n_trunc, rnd, pair.seed)
            assert list(g.get(binding.ARR_ORDER)) == order and np.array_equal(g.get(binding.ARR_DONOR), donor)
            assert int((donor >= 0).sum()) == wl.n_trunc
            after = {w: g.get(w) for w in arrays}
            for r in range(wl.P):
                src = donor[r] if donor[r] >= 0 else r
                for w in arrays:
                    if w != binding.ARR_HYPER:
                        assert after[w][r].tobytes() == before[w][src].tobytes(), (label, r, w)
                href = before[binding.ARR_HYPER][r] if donor[r] < 0 else opbt.perturb(
                    before[binding.ARR_HYPER][src], rnd, r, pair.seed, wl.perturb[0], wl.perturb[1], wl.h_max)
                assert after[binding.ARR_HYPER][r].tobytes() == href.tobytes(), (label, r)
            for i in sample:                       # an overwritten member restarts its free runs from the copy it received
                if donor[i] >= 0:
                    hs.sync_member(pair, free[i], i)
                    if near:
                        near[i] = _moved(free[i], rng)
            print(label, "exploit after step", s, "recipients in the sample:", [i for i in sample if donor[i] >= 0], "score", worst["score"], flush=True)
            rnd += 1
        if s % 10 == 9 or s == n_steps - 1:
            print(label, "step", s, {k: float("%.2g" % v) for k, v in worst.items()}, flush=True)
    print(label, "free-running drift (whole weight vector) after steps 1, 10, 25, 50, 100 and conditioning of the trajectory:")
    marks = [k for k in (0, 9, 24, 49, 99) if k < n_steps]
    for i in sample:
        print("   member %3d  h = %s  drift %s  conditioning %s" % (
            i, np.array2string(pair.gpu.get(binding.ARR_HYPER, i), precision=3), ["%.1e" % drift[i][k] for k in marks],
            ["%.1e" % cond[i][k] for k in marks] if near else "-"), flush=True)
    print(label, "free-running member-steps asserted against the tolerance:", n_asserted, "of", n_steps * len(sample), " window took %.0f s" % (time.time() - t_start), flush=True)
    return worst, drift, cond, n_asserted


def _spread(H, column, n):
    """n members spread over the quantiles of one hyperparameter column (smallest and largest included)."""
    order = np.argsort(H[:, column])
    return sorted({int(order[int(round(q * (len(order) - 1)))]) for q in np.linspace(0.0, 1.0, n)})


def test_mlp_wide_bf16_window():
    wl = workloads.MLP_WIDE
    sample = _spread(workloads.initial_hypers(wl, 6), 0, 6)
    pair = hs.Pair(wl, ref_members=sample)
    worst, drift, cond, n = run_window(pair, sample, 100, exploit_after=(50,), label="mlp_wide_bf16")
    assert n >= 100


def test_gan_mlp_bf16_window():
    wl = workloads.GAN_MLP
    sample = _spread(workloads.initial_hypers(wl, 6), 1, 4)
    pair = hs.GanPair(wl, ref_members=sample)
    worst, drift, cond, n = run_window(pair, sample, 100, exploit_after=(50,), label="gan_mlp_bf16")
    assert n >= 50


def test_a2c_mlp_bf16_window():
    wl = workloads.A2C_MLP
    sample = _spread(workloads.initial_hypers(wl, 6), 0, 8)
    pair = hs.A2CPair(wl, ref_members=sample)
    worst, drift, cond, n = run_window(pair, sample, 100, exploit_after=(50, 100), label="a2c_mlp_bf16")
    assert n >= 100


def test_transformer_bf16_window():
    """Full shape (P = 16, 21 M parameters per member), 10 steps with an eval + exploit/explore after step 5;
    two members followed per step and free-running (the held-out set is cut to 64 sequences so that the
    oracle's score stays affordable; the 256-sequence score is checked in test_gpu_transformer.py)."""
    wl = workloads.TRANSFORMER.replace(n_eval=64)
    H = workloads.initial_hypers(wl, 6)
    sample = sorted({int(np.argmax(H[:, 0])), int(np.argmin(H[:, 0]))})
    pair = hs.TransformerPair(wl, ref_members=sample)
    # Per parameter array the one-step weights are reported, not asserted: the member with the largest learning rate
    # (1e-3) moves every element by exactly lr in Adam's first steps, feed-forward matrices have an rms of 0.013, and
    # the gradient elements whose sign differs between fp32 and float64 accumulation of the same bf16 function (a few
    # percent: ReLU gates that flip move the gradients behind them) put single arrays at 2-3 %; the whole weight
    # vector stays within the tolerance.
    worst, drift, cond, n = run_window(pair, sample, 10, exploit_after=(5,), exact_at=(0, 9), with_conditioning=False,
                                       per_array=False, label="transformer_bf16")
    for i in sample:
        assert max(drift[i]) <= TOL, (i, drift[i])


def test_transformer_bf16_three_steps_all_members():
    """All 16 members free-running for three steps on both sides: every loss within the tolerance."""
    wl = workloads.TRANSFORMER
    pair = hs.TransformerPair(wl)
    worst = 0.0
    for s in range(3):
        pair.gpu.step(pair.d_pool, s)
        with threadpool_limits(limits=2):
            ref = np.array(list(_pool.map(lambda i: hs.oracle_step(pair, pair.ref[i], i, s)[0], range(wl.P))))
        worst = max(worst, _rel(pair.gpu.get(binding.ARR_LOSS), ref))
        assert worst <= TOL, (s, worst)
    print("transformer_bf16, 16 members x 3 free-running steps: worst loss error %.2e" % worst, flush=True)
