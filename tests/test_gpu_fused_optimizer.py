"""The optimiser applied inside the weight-gradient GEMMs (fuse_optimizer = 1) against the oracle and
against the separate optimiser pass, for all three optimisers and all bf16 workloads."""
import numpy as np
import pytest

from paper_1711_09846_amd import binding, workloads
from tests.harness import Pair, GanPair, A2CPair
from tests.test_gpu_classifier import _wide_reduced, _window, TOL_BF16
from tests.test_gpu_gan import _reduced as _gan_reduced
from tests.test_gpu_a2c import _reduced as _a2c_reduced

pytestmark = pytest.mark.gpu


def test_classifier_fused_window_against_oracle():
    pair = Pair(_wide_reduced(), eval_chunk=128, fuse_optimizer=1)
    _window(pair, 24, TOL_BF16, 8, opt1=True, verbose="mlp_wide_bf16 reduced, fused optimiser")


@pytest.mark.parametrize("make,cls,inputs", [(_wide_reduced, Pair, "d_train"), (_gan_reduced, GanPair, "d_train"),
                                              (_a2c_reduced, A2CPair, "d_pool")])
def test_fused_equals_separate_pass(make, cls, inputs):
    a, b = cls(make(), fuse_optimizer=0), cls(make(), fuse_optimizer=1)
    for s in range(6):
        a.gpu.step(getattr(a, inputs), s)
        b.gpu.step(getattr(b, inputs), s)
    arrays = [binding.ARR_W32, binding.ARR_OPT0] + ([binding.ARR_OPT1] if make().optimizer == workloads.OPT_ADAM else [])
    for which in arrays:
        x, y = a.gpu.get(which).astype(np.float64), b.gpu.get(which).astype(np.float64)
        # same arithmetic on the same gradient values; only the compiler's contraction choices may differ
        assert np.linalg.norm(x - y) <= 2e-6 * np.linalg.norm(x), which
    assert np.array_equal(a.gpu.get(binding.ARR_T), b.gpu.get(binding.ARR_T))
    la, lb = a.gpu.get(binding.ARR_LOSS), b.gpu.get(binding.ARR_LOSS)
    assert np.allclose(la, lb, rtol=1e-4, atol=1e-5)


def test_gan_fused_against_oracle():
    pair = GanPair(_gan_reduced(), fuse_optimizer=1)
    for s in range(8):
        pair.gpu.step(pair.d_train, s)
        pair.step_ref(s)
    for i in range(pair.wl.P):
        assert pair.member_errors(i, binding.ARR_W32, "theta")[0] <= TOL_BF16


def test_a2c_fused_against_oracle():
    pair = A2CPair(_a2c_reduced(), fuse_optimizer=1)
    for s in range(8):
        pair.gpu.step(pair.d_pool, s)
        pair.step_ref(s)
    for i in range(pair.wl.P):
        assert pair.member_errors(i, binding.ARR_W32, "theta")[0] <= TOL_BF16
        assert pair.member_errors(i, binding.ARR_OPT0, "s0")[1] <= TOL_BF16


def test_fused_full_size_against_separate_pass_and_oracle():
    """The wide workload at its real shape with the optimiser inside the weight-gradient GEMMs (the
    configuration the benchmark times): over 12 steps with an eval + exploit/explore after step 8 it
    follows the separate optimiser pass (same gradients, same update formula: the two may differ only in
    the compiler's contraction choices), and on every step a sample of members is re-synchronised and
    followed by the oracle for that step (whole parameter vector, optimiser state and loss)."""
    wl = workloads.MLP_WIDE.replace(ready_interval=8)
    sample = [0, 21, 63]
    a, b = Pair(wl, ref_members=[], fuse_optimizer=0), Pair(wl, ref_members=sample, fuse_optimizer=1)
    worst = dict(theta=0.0, s0=0.0, s1=0.0, loss=0.0)
    for s in range(12):
        for i in sample:
            b.sync_ref_from_gpu(i)
        a.gpu.step(a.d_train, s)
        b.gpu.step(b.d_train, s)
        loss_ref = b.step_ref(s)
        loss_gpu = b.gpu.get(binding.ARR_LOSS)[sample]
        worst["loss"] = max(worst["loss"], Pair.scalar_errors(loss_gpu, loss_ref, 1.0))
        for i in sample:
            for which, what in ((binding.ARR_W32, "theta"), (binding.ARR_OPT0, "s0"), (binding.ARR_OPT1, "s1")):
                worst[what] = max(worst[what], b.member_errors(i, which, what, rms_floor=1e-6 if what != "theta" else 0.0)[1])
        if s == 7:
            a.gpu.eval(a.d_eval); b.gpu.eval(b.d_eval)
            sa, sb = a.gpu.get(binding.ARR_SCORE), b.gpu.get(binding.ARR_SCORE)
            assert np.allclose(sa, sb, rtol=1e-4, atol=1e-5)
            a.gpu.exploit_explore(0); b.gpu.exploit_explore(0)
            if np.array_equal(np.argsort(-sa, kind="stable"), np.argsort(-sb, kind="stable")):
                assert np.array_equal(a.gpu.get(binding.ARR_PARENT), b.gpu.get(binding.ARR_PARENT))
                assert np.array_equal(a.gpu.get(binding.ARR_HYPER), b.gpu.get(binding.ARR_HYPER))
            else:  # a rounding-level score difference reordered two members: continue from the same state
                for which in (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_OPT1, binding.ARR_HYPER, binding.ARR_T):
                    b.gpu.set(which, a.gpu.get(which))
    print("fused, full size: worst per-step distance to the oracle", worst)
    assert worst["theta"] <= TOL_BF16 and worst["s0"] <= TOL_BF16 and worst["s1"] <= TOL_BF16 and worst["loss"] <= TOL_BF16
    for which in (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_OPT1):
        x, y = a.gpu.get(which).astype(np.float64), b.gpu.get(which).astype(np.float64)
        for i in range(wl.P):
            assert np.linalg.norm(x[i] - y[i]) <= 1e-5 * np.linalg.norm(x[i]), (which, i)
    assert np.array_equal(a.gpu.get(binding.ARR_T), b.gpu.get(binding.ARR_T))
