"""Device-side initial population against the oracle's."""
import numpy as np
import pytest

from oracle import pbt as opbt
from paper_1711_09846_amd import binding, workloads

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("key", [1, 2])
def test_init_population_matches_oracle(key):
    wl = workloads.WORKLOADS[key].replace(P=6, n_trunc=1)
    seed = 0x1234567_89abcdef
    pop = binding.Population(binding.make_config(wl, seed))
    pop.set(binding.ARR_T, np.full(wl.P, 9, dtype=np.int32))       # must be reset by the init
    pop.init_population(wl.priors)
    lay = pop.layout
    offsets = [(lay.w_off[l], lay.b_off[l]) for l in range(len(wl.dims) - 1)]
    W = pop.get(binding.ARR_W32)
    for i in range(wl.P):
        ref = binding.pack_params(lay, opbt.init_weights(seed, i, wl.dims, offsets))
        assert W[i].tobytes() == ref.tobytes()                    # division and sqrt are correctly rounded on both sides
    H, Href = pop.get(binding.ARR_HYPER), opbt.init_hyperparameters(seed, wl.P, wl.priors)
    # exp() may differ by an ulp of double between the two math libraries; after rounding to float
    # that can at most move the result to the neighbouring float
    assert np.all(np.abs(H.view(np.int32) - Href.view(np.int32)) <= 1)
    assert np.array_equal(H[:, 1:], Href[:, 1:]) or key == 2
    assert np.all(pop.get(binding.ARR_T) == 0) and np.all(pop.get(binding.ARR_OPT0) == 0)
    assert np.array_equal(pop.get(binding.ARR_PARENT), np.arange(wl.P))
    if wl.dtype == workloads.DTYPE_BF16:
        import torch
        w16 = torch.from_numpy(W).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(pop.get(binding.ARR_W16), w16)


def test_init_population_rejects_bad_priors():
    pop = binding.Population(binding.make_config(workloads.MLP_SMALL, 1))
    with pytest.raises(binding.PbtError):
        pop.init_population([("log", 0.0, 1.0)])
    with pytest.raises(binding.PbtError):
        pop.init_population([("uniform", 2.0, 1.0)])


def test_init_population_transformer_matches_oracle():
    from oracle import transformer as ot
    wl = workloads.TRANSFORMER.replace(P=3, vocab=64, d_model=32, heads=2, d_ff=64, n_blocks=2, seq=16, batch=4, n_train=64, n_eval=8, n_trunc=1)
    seed = 0x51
    pop = binding.Population(binding.make_config(wl, seed))
    pop.init_population(wl.priors)
    lay = pop.layout
    spec = ot.TransformerSpec(wl.vocab, wl.d_model, wl.heads, wl.d_ff, wl.n_blocks, wl.seq, wl.batch, seed, roles=wl.roles)
    shapes = workloads.transformer_shapes(wl)
    W, W16 = pop.get(binding.ARR_W32), pop.get(binding.ARR_W16)
    for i in range(wl.P):
        ref = binding.pack_segments(lay, ot.init_arrays(spec, seed, i, [lay.seg_off[j] for j in range(lay.n_seg)]))
        assert W[i].tobytes() == ref.tobytes()
        got = binding.unpack_segments(lay, shapes, W[i])
        assert np.all(got[2] == 1.0) and np.all(got[3] == 0.0) and np.all(got[-1] == 0.0)     # gain, bias, head bias
    import torch
    assert np.array_equal(W16, torch.from_numpy(W).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    H, Href = pop.get(binding.ARR_HYPER), opbt.init_hyperparameters(seed, wl.P, wl.priors)
    assert np.all(np.abs(H.view(np.int32) - Href.view(np.int32)) <= 1)
    # and the initialised population trains
    pair_pool, _ = workloads.zipf_bigram_sequences(wl)
    d_pool = [torch.from_numpy(pair_pool).cuda()]
    pop.step(d_pool, 0)
    l0 = pop.get(binding.ARR_LOSS).copy()
    for s in range(1, 40):
        pop.step(d_pool, s)
    assert np.all(np.isfinite(l0)) and np.all(pop.get(binding.ARR_LOSS) < l0)


def test_init_population_gan_two_networks_match_oracle():
    """Generator and discriminator live in one flat vector; every layer of both is drawn with its own fan-in."""
    wl = workloads.GAN_MLP.replace(P=4, dims=[16, 72, 40], dims2=[40, 136, 24, 1], batch=24, n_train=1024, n_eval=200, n_trunc=1)
    seed = 0x77aa
    pop = binding.Population(binding.make_config(wl, seed))
    pop.init_population(wl.priors)
    lay = pop.layout
    Lg, Ld = len(wl.dims) - 1, len(wl.dims2) - 1
    off_g = [(lay.w_off[l], lay.b_off[l]) for l in range(Lg)]
    off_d = [(lay.w_off[Lg + l], lay.b_off[Lg + l]) for l in range(Ld)]
    W = pop.get(binding.ARR_W32)
    for i in range(wl.P):
        layers = opbt.init_weights(seed, i, wl.dims, off_g) + opbt.init_weights(seed, i, wl.dims2, off_d)
        assert W[i].tobytes() == binding.pack_params(lay, layers).tobytes()
        # the first discriminator layer really uses its own fan-in (40), not the generator's
        Wd0 = W[i][lay.w_off[Lg]:lay.w_off[Lg] + 40 * 136]
        assert 0.9 / np.sqrt(40) < np.abs(Wd0).max() <= 1.0 / np.sqrt(40)
    H, Href = pop.get(binding.ARR_HYPER), opbt.init_hyperparameters(seed, wl.P, wl.priors)
    assert np.all(np.abs(H.view(np.int32) - Href.view(np.int32)) <= 1)
    import torch
    assert np.array_equal(pop.get(binding.ARR_W16), torch.from_numpy(W).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
