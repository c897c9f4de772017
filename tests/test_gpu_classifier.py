"""The population step (`step`, `eval`, exploit/explore) of the classifier workloads on the GPU
against the oracle: weights, optimiser state, losses and scores within the stated tolerance at
every step of a free-running window; selection bit-exact given the same scores."""
import numpy as np
import pytest

from paper_1711_09846_amd import binding, workloads
from tests.harness import Pair

pytestmark = pytest.mark.gpu

TOL_FP32 = 1e-5     # relative, fp32 compute
TOL_BF16 = 1e-2     # relative, bf16 compute with fp32 master weights
# Losses and scores are compared as |gpu - ref| / max(|ref|, floor).  A loss is lse(logits) minus the
# label's logit: its absolute error is set by the rounding of O(10) logits and does not shrink with
# the loss, so a purely relative test is unattainable in any finite precision once training drives
# the loss towards 0.  fp32: floor 1e-3.  bf16: logits carry 2^-9 relative rounding; floor 0.1 (measured
# absolute errors stay below 1e-4 while the logits grow past 1000).
FLOOR_FP32 = 1e-3
FLOOR_BF16 = 0.1


def _window(pair, n_steps, tol, ready_interval, check_every=1, opt1=False, verbose="", tol_scalar=None):
    tol_scalar = tol if tol_scalar is None else tol_scalar
    floor = FLOOR_BF16 if pair.wl.dtype == workloads.DTYPE_BF16 else FLOOR_FP32
    worst = dict(w=0.0, s0=0.0, s1=0.0, loss=0.0, score=0.0)
    rnd = 0
    for s in range(n_steps):
        pair.gpu.step(pair.d_train, s)
        loss_ref = pair.step_ref(s)
        if (s + 1) % check_every == 0 or s == n_steps - 1:
            worst["loss"] = max(worst["loss"], pair.scalar_errors(pair.gpu.get(binding.ARR_LOSS), loss_ref, floor))
            worst["w"] = max(worst["w"], pair.tensor_errors(binding.ARR_W32, "theta"))
            worst["s0"] = max(worst["s0"], pair.tensor_errors(binding.ARR_OPT0, "s0"))
            if opt1:
                worst["s1"] = max(worst["s1"], pair.tensor_errors(binding.ARR_OPT1, "s1"))
            assert worst["w"] <= tol and worst["loss"] <= tol_scalar, (s, worst, loss_ref)
        if ready_interval and (s + 1) % ready_interval == 0:
            pair.gpu.eval(pair.d_eval)
            sc_gpu = pair.gpu.get(binding.ARR_SCORE)
            sc_ref = pair.eval_ref()
            worst["score"] = max(worst["score"], pair.scalar_errors(sc_gpu, sc_ref, floor))
            assert worst["score"] <= tol_scalar, (s, worst, sc_ref)
            # both sides rank the same (GPU) score vector
            pair.gpu.exploit_explore(rnd)
            order, donor = pair.exploit_ref(rnd, sc_gpu)
            assert list(pair.gpu.get(binding.ARR_ORDER)) == order
            assert np.array_equal(pair.gpu.get(binding.ARR_DONOR), donor)
            assert pair.gpu.get(binding.ARR_HYPER).tobytes() == np.stack([m.h for m in pair.ref]).tobytes()
            rnd += 1
    print(verbose, "worst relative errors:", {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)
    return worst


def test_mlp_small_fp32_100_steps():
    """Two-layer fp32 MLPs, SGD momentum, P = 8, exploit every 50 steps."""
    pair = Pair(workloads.MLP_SMALL)
    w = _window(pair, 100, TOL_FP32, workloads.MLP_SMALL.ready_interval, verbose="mlp_small_fp32")
    assert w["s0"] <= 1e-4


def test_mlp_small_fp32_multi_step_launch_equals_single_steps():
    a, b = Pair(workloads.MLP_SMALL), Pair(workloads.MLP_SMALL)
    for s in range(10):
        a.gpu.step(a.d_train, s)
    b.gpu.step(b.d_train, 0, n_steps=10)
    for which in (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_T, binding.ARR_LOSS):
        assert a.gpu.get(which).tobytes() == b.gpu.get(which).tobytes()


@pytest.mark.parametrize("opt", [workloads.OPT_ADAM, workloads.OPT_RMSPROP, workloads.OPT_SGD_MOMENTUM])
def test_fp32_other_optimizers(opt):
    roles = [workloads.ROLE_LR, workloads.ROLE_BETA1, workloads.ROLE_WD] if opt == workloads.OPT_ADAM else [workloads.ROLE_LR]
    priors = [("log", 1e-3, 1e-2), ("uniform", 0.8, 0.95), ("log", 1e-6, 1e-3)][:len(roles)]
    oc = {workloads.OPT_ADAM: dict(beta2=0.999, eps=1e-8), workloads.OPT_RMSPROP: dict(rho=0.99, eps=1e-5),
          workloads.OPT_SGD_MOMENTUM: dict(momentum=0.9)}[opt]
    wl = workloads.MLP_SMALL.replace(optimizer=opt, roles=roles, priors=priors, h_max=[np.inf, 0.999, np.inf][:len(roles)],
                                     opt_const=oc, dims=[32, 24, 40, 4], act=workloads.ACT_GELU, P=5, n_trunc=1)
    pair = Pair(wl)
    # Not one of the named workloads: Adam drives these losses below 1e-2, where the loss is a
    # difference of O(10) logits and fp32 rounding of the logits bounds its relative accuracy.
    _window(pair, 30, 2e-5, 10, opt1=opt == workloads.OPT_ADAM, verbose="fp32 opt %d" % opt, tol_scalar=2e-4)


def _wide_reduced(P=6):
    # same structure as the wide workload, dims spanning several MFMA tiles with ragged tails
    # (lr prior capped at 3e-3: on this tiny data set larger Adam rates diverge, and a diverging
    # member amplifies any rounding difference without bound)
    return workloads.MLP_WIDE.replace(P=P, dims=[72, 200, 136, 10], batch=40, n_train=4096, n_eval=300, n_trunc=1,
                                      ready_interval=8,
                                      priors=[("log", 1e-4, 3e-3), ("uniform", 0.8, 0.95), ("log", 1e-6, 1e-3)])


def test_mlp_wide_bf16_reduced_window():
    pair = Pair(_wide_reduced(), eval_chunk=128)
    _window(pair, 24, TOL_BF16, 8, opt1=True, verbose="mlp_wide_bf16 reduced")


def test_bf16_gradients_one_step():
    """Teacher-forced single step: gradient buffer against the oracle's gradient."""
    from oracle import nets, classifier as oc
    pair = Pair(_wide_reduced(P=3))
    pair.gpu.step(pair.d_train, 0)
    G = pair.gpu.get(binding.ARR_GRAD).astype(np.float64)
    lay, dims = pair.gpu.layout, pair.wl.dims
    for i, m in enumerate(pair.ref):
        rows = oc.batch_rows(pair.seed, 0, i, pair.wl.batch, len(pair.train_y))
        _, grads = nets.classifier_loss_and_grads(oc.params_of(m), pair.train_x[rows], pair.train_y[rows], pair.wl.act)
        for l, (gW, gb) in enumerate(grads):
            g = G[i, lay.w_off[l]:lay.w_off[l] + gW.size].reshape(gW.shape)
            assert np.linalg.norm(g - gW) / np.linalg.norm(gW) < 1e-2, (i, l)
            g = G[i, lay.b_off[l]:lay.b_off[l] + gb.size]
            assert np.linalg.norm(g - gb) / np.linalg.norm(gb) < 1e-2, (i, l)


def test_member_independence_bitwise():
    """Without exploit a member's trajectory does not depend on who else is in the population."""
    wl = _wide_reduced(P=4)
    full = Pair(wl)
    for s in range(5):
        full.gpu.step(full.d_train, s)
    # same member 2, but the other members' weights and hyperparameters are different
    other = Pair(wl, init_seed=77)
    other.gpu.set(binding.ARR_W32, full_initial(full, 2), member=2)
    other.gpu.set(binding.ARR_HYPER, workloads.initial_hypers(wl, 6)[2], member=2)
    for s in range(5):
        other.gpu.step(other.d_train, s)
    assert full.gpu.get(binding.ARR_W32, 2).tobytes() == other.gpu.get(binding.ARR_W32, 2).tobytes()


def full_initial(pair, member):
    weights = workloads.initial_mlp_weights(pair.wl.dims, pair.wl.P, 5)
    return binding.pack_params(pair.gpu.layout, weights[member])


def _flatten_grads(pair, grads):
    lay = pair.gpu.layout
    flat = np.zeros(lay.stride)
    for l, (gW, gb) in enumerate(grads):
        flat[lay.w_off[l]:lay.w_off[l] + gW.size] = gW.ravel()
        flat[lay.b_off[l]:lay.b_off[l] + gb.size] = gb
    return flat


def test_mlp_wide_bf16_full_size_window():
    """The wide workload at its real shape (P = 64, 256-1024-1024-10, batch 128, Adam), 100 steps
    with an eval + exploit/explore after step 50, all 64 members on the GPU.  A sample of members
    (largest and smallest learning rate plus seeded picks) is followed by the oracle one by one.

    Per step, from the GPU's state at the start of the step (the oracle is re-synchronised, so the
    bound is on what one step adds): (a) the gradient, (b) the optimiser update given the GPU's own
    gradient, at fp32 accuracy, (c) loss and the whole updated parameter vector.
    (a) is asserted while the member's loss is >= 1e-3, see below.  Splitting (a)
    from (b) keeps both well conditioned: Adam's update lr*m/(sqrt(v)+eps) has slope lr/eps = 1e6
    in g where |g| ~ eps, so a handful of elements with |g| ~ 1e-8 move by up to lr under a 1e-5
    relative change of the gradient; that is a property of the formula, not of an implementation.
    A second set of oracle twins runs free between exploit points; its drift is reported and
    bounded at the median (single members that train into saturation amplify any rounding
    difference without bound)."""
    import copy
    from oracle import nets, classifier as oc, pbt as opbt
    wl = workloads.MLP_WIDE.replace(ready_interval=50)
    H0 = workloads.initial_hypers(wl, 6)
    rng = np.random.default_rng(3)
    sample = sorted(set([int(np.argmax(H0[:, 0])), int(np.argmin(H0[:, 0]))] + [int(v) for v in rng.choice(wl.P, 6, replace=False)]))
    pair = Pair(wl, ref_members=sample)
    assert np.array_equal(pair.gpu.get(binding.ARR_HYPER), H0)
    free = {i: copy.deepcopy(pair.ref[i]) for i in sample}
    worst = dict(grad=0.0, opt=0.0, step=0.0, loss=0.0, score=0.0, drift_median=0.0, drift_max=0.0)
    g = pair.gpu
    n_grad_checks = 0
    for s in range(100):
        for i in sample:
            pair.sync_ref_from_gpu(i)
        g.step(pair.d_train, s)
        loss_gpu = g.get(binding.ARR_LOSS)
        drifts = []
        for i in sample:
            m = pair.ref[i]
            rows = oc.batch_rows(pair.seed, s, i, wl.batch, wl.n_train)
            loss_ref, grads = nets.classifier_loss_and_grads(oc.params_of(m), pair.train_x[rows], pair.train_y[rows],
                                                             wl.act, pair.spec.q)
            worst["loss"] = max(worst["loss"], abs(loss_gpu[i] - loss_ref) / max(abs(loss_ref), FLOOR_BF16))
            # (a) gradient, while the member's loss is >= 1e-3.  Below that every softmax term
            # e^(l_c - l_y) turns the absolute fp32 rounding of the logits (which grows with their
            # size, > 1000 here for members trained into saturation) into relative error of the
            # gradient; there the gradient is only judged through the weights it produces, (c).
            if loss_ref >= 1e-3:
                n_grad_checks += 1
                worst["grad"] = max(worst["grad"], pair.member_errors(i, binding.ARR_GRAD, None,
                                                                      _flatten_grads(pair, grads))[0])
            # (b) optimiser on the GPU's gradient
            g_gpu = binding.unpack_params(g.layout, wl.dims, g.get(binding.ARR_GRAD, i).astype(np.float64))
            m_b = copy.deepcopy(m)
            oc.apply_optimizer(pair.spec, m_b, [a for Wb in g_gpu for a in Wb])
            keep, pair.ref[i] = pair.ref[i], m_b
            for which, what in ((binding.ARR_W32, "theta"), (binding.ARR_OPT0, "s0"), (binding.ARR_OPT1, "s1")):
                worst["opt"] = max(worst["opt"], pair.member_errors(i, which, what)[0])
            pair.ref[i] = keep
            # (c) the whole step with the oracle's own gradient
            oc.apply_optimizer(pair.spec, m, [a for gr in grads for a in gr])
            worst["step"] = max(worst["step"], pair.member_errors(i, binding.ARR_W32, "theta")[1])
            assert int(g.get(binding.ARR_T, i)[0]) == m.t
            # free-running twin
            oc.step(pair.spec, free[i], i, s, pair.train_x, pair.train_y)
            keep, pair.ref[i] = pair.ref[i], free[i]
            drifts.append(pair.member_errors(i, binding.ARR_W32, "theta")[1])
            pair.ref[i] = keep
        worst["drift_median"] = max(worst["drift_median"], float(np.median(drifts)))
        worst["drift_max"] = max(worst["drift_max"], float(np.max(drifts)))
        assert worst["grad"] <= TOL_BF16 and worst["opt"] <= TOL_FP32 and worst["step"] <= TOL_BF16 \
            and worst["loss"] <= TOL_BF16 and worst["drift_median"] <= TOL_BF16, (s, worst)
        if s % 10 == 9:
            print("step", s, {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)
        if s == 49:
            g.eval(pair.d_eval)
            sc_gpu = g.get(binding.ARR_SCORE)
            for i in sample:
                pair.sync_ref_from_gpu(i)
            sc_ref = pair.eval_ref()
            worst["score"] = pair.scalar_errors(sc_gpu[sample], sc_ref, FLOOR_BF16)
            assert worst["score"] <= TOL_BF16, worst
            before = {w: g.get(w) for w in (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_OPT1, binding.ARR_W16,
                                            binding.ARR_HYPER, binding.ARR_T)}
            g.exploit_explore(0)
            order, donor = opbt.truncation_select(sc_gpu, wl.n_trunc, 0, pair.seed)
            assert list(g.get(binding.ARR_ORDER)) == order and np.array_equal(g.get(binding.ARR_DONOR), donor)
            assert (donor >= 0).sum() == wl.n_trunc
            after = {w: g.get(w) for w in before}
            for r in range(wl.P):
                src = donor[r] if donor[r] >= 0 else r
                for w in (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_OPT1, binding.ARR_W16, binding.ARR_T):
                    assert after[w][r].tobytes() == before[w][src].tobytes(), (r, w)
                href = before[binding.ARR_HYPER][r] if donor[r] < 0 else opbt.perturb(
                    before[binding.ARR_HYPER][src], 0, r, pair.seed, wl.perturb[0], wl.perturb[1], wl.h_max)
                assert after[binding.ARR_HYPER][r].tobytes() == href.tobytes(), r
            for i in sample:                       # recipients restart their free run from the copy
                if donor[i] >= 0:
                    pair.sync_ref_from_gpu(i)
                    free[i] = copy.deepcopy(pair.ref[i])
    assert n_grad_checks >= 100, n_grad_checks
    print("mlp_wide_bf16 full size:", {k: float("%.3g" % v) for k, v in worst.items()}, "gradient checks:", n_grad_checks, flush=True)
