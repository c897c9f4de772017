"""pbt_step_static (the step with the library's static working memory, for callers that cannot
allocate) against pbt_step: same kernels, so every array of the population store must come out
bit-identical, on two calls in a row that share the static array, the second with a smaller input."""
import numpy as np
import pytest

from paper_1711_09846_amd import binding, workloads
from tests.harness import Pair

pytestmark = pytest.mark.gpu

ARRAYS_BF16 = (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_OPT1, binding.ARR_W16, binding.ARR_T, binding.ARR_LOSS)
ARRAYS_FP32 = (binding.ARR_W32, binding.ARR_OPT0, binding.ARR_T, binding.ARR_LOSS)


def _bigger():
    return workloads.MLP_WIDE.replace(P=6, dims=[72, 200, 136, 10], batch=40, n_train=4096, n_eval=300, n_trunc=1,
                                      priors=[("log", 1e-4, 3e-3), ("uniform", 0.8, 0.95), ("log", 1e-6, 1e-3)])


def _smaller():
    return workloads.MLP_WIDE.replace(P=3, dims=[40, 64, 10], batch=24, n_train=1024, n_eval=100, n_trunc=1,
                                      priors=[("log", 1e-4, 3e-3), ("uniform", 0.8, 0.95), ("log", 1e-6, 1e-3)])


def _same(a, b, arrays):
    for which in arrays:
        assert a.gpu.get(which).tobytes() == b.gpu.get(which).tobytes(), which


def test_static_step_equals_step_on_two_calls_the_second_smaller():
    # call 1: the bigger population fills the static array with its gradients and activations
    a, b = Pair(_bigger(), eval_chunk=128), Pair(_bigger(), eval_chunk=128)
    assert a.gpu.scratch.numel() <= binding.STATIC_SCRATCH_BYTES
    a.gpu.step(a.d_train, 0)
    b.gpu.step_static(b.d_train, 0)
    _same(a, b, ARRAYS_BF16)
    # call 2, straight after it: a smaller population, whose buffers now overlay what call 1 left behind
    c, d = Pair(_smaller()), Pair(_smaller())
    c.gpu.step(c.d_train, 0)
    d.gpu.step_static(d.d_train, 0)
    _same(c, d, ARRAYS_BF16)
    # and both keep agreeing over further alternating calls (padding of theta stays zero on both sides)
    for s in range(1, 4):
        a.gpu.step(a.d_train, s)
        b.gpu.step_static(b.d_train, s)
        c.gpu.step(c.d_train, s)
        d.gpu.step_static(d.d_train, s)
    _same(a, b, ARRAYS_BF16)
    _same(c, d, ARRAYS_BF16)
    lay = b.gpu.layout
    pad = np.ones(lay.stride, dtype=bool)
    for j in range(lay.n_seg):
        pad[lay.seg_off[j]:lay.seg_off[j] + lay.seg_len[j]] = False
    assert not np.any(b.gpu.get(binding.ARR_W32)[:, pad])
    # the scores that follow from those weights agree too
    a.gpu.eval(a.d_eval)
    b.gpu.eval(b.d_eval)
    assert a.gpu.get(binding.ARR_SCORE).tobytes() == b.gpu.get(binding.ARR_SCORE).tobytes()


def test_static_step_fp32_multi_step_launch():
    a, b = Pair(workloads.MLP_SMALL), Pair(workloads.MLP_SMALL)
    a.gpu.step(a.d_train, 0, n_steps=7)
    b.gpu.step_static(b.d_train, 0, n_steps=7)
    _same(a, b, ARRAYS_FP32)


def test_static_step_rejects_what_does_not_fit():
    """The full-size wide workload needs ~1 GB of working memory: refused with a clear error before any launch."""
    pop = binding.Population(binding.make_config(workloads.MLP_WIDE, 1))
    (tx, ty), _ = workloads.classifier_data(workloads.MLP_WIDE.replace(n_train=256, n_eval=16))
    import torch
    d = [torch.from_numpy(tx).to(pop.device), torch.from_numpy(ty).to(pop.device)]
    before = pop.get(binding.ARR_T).copy()
    with pytest.raises(binding.PbtError) as e:
        pop.step_static(d, 0)
    assert e.value.status == -2 and "static" in str(e.value)
    assert np.array_equal(pop.get(binding.ARR_T), before)
