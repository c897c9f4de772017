"""Host-side checks of the C-ABI library (no GPU needed): it loads, exports every symbol the header
declares, lays parameters out as documented and rejects bad configurations before touching a device."""
import math
import os
import re

import numpy as np
import pytest

from paper_1711_09846_amd import binding, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(binding.LIB_PATH):
        from paper_1711_09846_amd import build
        build.build_library(verbose=False)


def test_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pbt.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(pbt_[a-z0-9_]+)\s*\(", header))
    assert {"pbt_init", "pbt_step", "pbt_eval", "pbt_exploit_explore", "pbt_get_state"} <= declared
    lib = binding.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding.EXPORTS)


def test_layout_and_sizes():
    for key, n_params in ((1, 2372), (2, 1323018)):
        wl = workloads.WORKLOADS[key]
        cfg = binding.make_config(wl, 1)
        state, scratch, lay = binding.query_sizes(cfg)
        assert lay.n_params == n_params and lay.stride % 256 == 0 and lay.stride >= n_params
        off = 0
        for l, (fi, fo) in enumerate(zip(wl.dims[:-1], wl.dims[1:])):
            assert lay.w_off[l] % 64 == 0 and lay.b_off[l] % 64 == 0
            assert lay.w_off[l] >= off and lay.b_off[l] >= lay.w_off[l] + fi * fo
            off = lay.b_off[l] + fo
        n_arrays = {1: 2, 2: 3}[key]
        assert state >= wl.P * lay.stride * 4 * n_arrays and scratch >= wl.P * lay.stride * 4


def test_pack_unpack_roundtrip():
    wl = workloads.MLP_SMALL
    _, _, lay = binding.query_sizes(binding.make_config(wl, 1))
    layers = workloads.initial_mlp_weights(wl.dims, 1, 0)[0]
    flat = binding.pack_params(lay, layers)
    assert flat.shape == (lay.stride,) and np.count_nonzero(flat) <= lay.n_params
    for (W, b), (W2, b2) in zip(layers, binding.unpack_params(lay, wl.dims, flat)):
        assert np.array_equal(W, W2) and np.array_equal(b, b2)


@pytest.mark.parametrize("change,status", [
    (dict(P=0), -1), (dict(P=2000), -1), (dict(n_trunc=5), -1), (dict(batch=0), -1),
    (dict(roles=[workloads.ROLE_BETA1]), -1),                     # no learning-rate column
    (dict(kind=7), -5),                                           # workload family not built
    (dict(dims=[32, 64, 40]), -5),                                # more than 32 classes
    (dict(dims=[32, 4096, 4096, 4]), -5),                         # fp32 network that does not fit LDS
])
def test_bad_configurations_are_rejected(change, status):
    wl = workloads.MLP_SMALL.replace(**change)
    if "roles" in change:
        wl = wl.replace(priors=[("uniform", 0.8, 0.9)], h_max=[math.inf], optimizer=workloads.OPT_ADAM,
                        opt_const=dict())
    with pytest.raises(binding.PbtError) as e:
        binding.query_sizes(binding.make_config(wl, 1))
    assert e.value.status == status and len(str(e.value)) > 20


def test_trunc_count_rule():
    assert [workloads.trunc_count(P, pc) for P, pc in ((8, 25), (64, 20), (32, 20), (16, 20), (128, 20), (3, 20))] == \
        [2, 12, 6, 3, 25, 1]


def test_transformer_layout_lists_every_parameter_array_in_order():
    wl = workloads.TRANSFORMER
    state, scratch, lay = binding.query_sizes(binding.make_config(wl, 1))
    shapes = workloads.transformer_shapes(wl)
    assert lay.n_seg == len(shapes) == 2 + 12 * wl.n_blocks + 4
    sizes = [int(np.prod(s)) for s in shapes]
    assert [lay.seg_len[j] for j in range(lay.n_seg)] == sizes and lay.n_params == sum(sizes)
    end = 0
    for j in range(lay.n_seg):
        assert lay.seg_off[j] >= end and lay.seg_off[j] % 8 == 0      # no overlap, 16-byte aligned as bf16
        end = lay.seg_off[j] + lay.seg_len[j]
    assert end <= lay.stride
    assert state >= wl.P * lay.stride * (4 * 3 + 2) and scratch > wl.P * lay.stride * 4
    arrays = workloads.initial_transformer_weights(wl.replace(vocab=64, d_model=16, heads=2, d_ff=32, seq=8, n_blocks=1), 1, 3)[0]
    small = binding.query_sizes(binding.make_config(wl.replace(vocab=64, d_model=16, heads=2, d_ff=32, seq=8, n_blocks=1), 1))[2]
    flat = binding.pack_segments(small, arrays)
    back = binding.unpack_segments(small, [a.shape for a in arrays], flat)
    assert all(np.array_equal(a, b) for a, b in zip(arrays, back))


@pytest.mark.parametrize("change", [dict(d_model=500), dict(heads=3), dict(seq=100), dict(n_eval=250), dict(h_max=[math.inf, 1.0, 0.9]),
                                    dict(optimizer=workloads.OPT_RMSPROP, opt_const=dict(rho=0.9, eps=1e-5)),
                                    dict(seq=4104, batch=1, n_eval=1), dict(seq=1024, batch=16, n_eval=16)])
def test_transformer_bad_configurations_are_rejected(change):
    cfg = binding.make_config(workloads.TRANSFORMER.replace(**change), 1)
    with pytest.raises(binding.PbtError):
        binding.query_sizes(cfg)


def test_dense_workload_segments_mirror_layer_offsets():
    _, _, lay = binding.query_sizes(binding.make_config(workloads.MLP_WIDE, 1))
    dims = workloads.MLP_WIDE.dims
    assert lay.n_seg == 2 * (len(dims) - 1)
    for l in range(len(dims) - 1):
        assert (lay.seg_off[2 * l], lay.seg_len[2 * l]) == (lay.w_off[l], dims[l] * dims[l + 1])
        assert (lay.seg_off[2 * l + 1], lay.seg_len[2 * l + 1]) == (lay.b_off[l], dims[l + 1])


@pytest.mark.parametrize("bad", [dict(exploit_mode=3), dict(explore_mode=5), dict(resample_prob=-0.5), dict(keep_weights=1, keep_hypers=1),
                                 dict(exploit_mode=2, ttest_alpha=0.05)])
def test_exploit_variant_configurations_are_checked(bad):
    """The last case: t-test selection needs the actor-critic workload's score history."""
    with pytest.raises(binding.PbtError):
        binding.query_sizes(binding.make_config(workloads.MLP_WIDE.replace(**bad), 1))


def test_exploit_variants_size_their_staging_rows():
    base = binding.query_sizes(binding.make_config(workloads.MLP_WIDE, 1))
    tour = binding.query_sizes(binding.make_config(workloads.MLP_WIDE.replace(exploit_mode=1), 1))
    assert tour[0] == base[0] and tour[1] >= base[1] + workloads.MLP_WIDE.P * base[2].stride * 14
    ok = binding.query_sizes(binding.make_config(workloads.A2C_MLP.replace(exploit_mode=2, ttest_alpha=0.05), 1))
    assert ok[1] > binding.query_sizes(binding.make_config(workloads.A2C_MLP, 1))[1]
    for alpha in (0.0, 1.5):
        with pytest.raises(binding.PbtError):
            binding.query_sizes(binding.make_config(workloads.A2C_MLP.replace(exploit_mode=2, ttest_alpha=alpha), 1))


def test_actor_critic_rejects_optimizers_it_has_no_state_for():
    """The actor-critic step hands one optimiser-state array to the update kernels: Adam is refused at
    configuration time (both by the size query and, through the same check, by pbt_init)."""
    for opt, oc in ((workloads.OPT_RMSPROP, dict(rho=0.99, eps=1e-5)), (workloads.OPT_SGD_MOMENTUM, dict(momentum=0.9))):
        binding.query_sizes(binding.make_config(workloads.A2C_MLP.replace(optimizer=opt, opt_const=oc), 1))
    with pytest.raises(binding.PbtError) as e:
        binding.query_sizes(binding.make_config(workloads.A2C_MLP.replace(optimizer=workloads.OPT_ADAM, opt_const=dict()), 1))
    assert e.value.status == -5


def test_beta1_column_needs_an_upper_clamp_below_one():
    """Explore only clamps at hyper_max; beta1 >= 1 would make Adam's bias correction infinite."""
    binding.query_sizes(binding.make_config(workloads.MLP_WIDE, 1))
    for bad in (1.0, math.inf):
        with pytest.raises(binding.PbtError) as e:
            binding.query_sizes(binding.make_config(workloads.MLP_WIDE.replace(h_max=[math.inf, bad, math.inf]), 1))
        assert e.value.status == -1
