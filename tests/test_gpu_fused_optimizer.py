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
