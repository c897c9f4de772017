"""The language-model workload on the GPU against the oracle: embeddings, pre-LayerNorm blocks with
causal attention, Philox dropout at four sites per block, label-smoothed cross-entropy, Adam, and the
perplexity score (Section 4.2.1)."""
import numpy as np
import pytest

from paper_1711_09846_amd import binding, workloads
from tests.harness import TransformerPair

pytestmark = pytest.mark.gpu

TOL_BF16 = 1e-2
FLOOR = 1e-2    # |gpu - ref| / max(|ref|, FLOOR) for the loss (ln V = 9 at the start)
# Gradients of the reduced networks: where no stored bf16 value rounds differently under fp32 and fp64
# accumulation the two sides agree to ~1e-7; one value rounding the other way (about two are expected
# per forward pass of these sizes) moves every gradient of a 64-row batch by up to a few percent (the
# oracle's own gradients move by 3-12 % when bf16 storage is switched on).  So: every case within
# TOL_GRAD_SMALL, and a good share of them essentially exact.
TOL_GRAD_SMALL = 5e-2
EXACT = 1e-5
# Weights are compared per parameter array relative to the array's norm, but at no smaller scale than
# an rms of W_FLOOR (a tenth of the initial weight scale): the biases start at zero and are a few
# learning rates long after a few steps, where "relative error of the weights" would just repeat the
# relative error of the gradient.
W_FLOOR = 1e-2


def _reduced(P=3, **kw):
    base = dict(P=P, vocab=64, d_model=32, heads=2, d_ff=64, n_blocks=2, seq=16, batch=4, n_train=64, n_eval=8, n_trunc=1)
    base.update(kw)
    return workloads.TRANSFORMER.replace(**base)


def _teacher_forced(pair, steps, members, grad_floor=0.0, tol_grad=TOL_GRAD_SMALL, tol_w=TOL_BF16):
    """Before every step the oracle takes over the GPU's state; compares the loss, the gradient of
    every parameter array and the updated weights of that one step."""
    g, ot = pair.gpu, pair.ot
    worst = dict(loss=0.0, grad=0.0, step=0.0, s0=0.0, s1=0.0)
    cases = []
    names = [n for n, _ in pair.spec.param_shapes()]
    for s in steps:
        for i in members:
            pair.sync_ref_from_gpu(i)
        g.step(pair.d_pool, s)
        loss = g.get(binding.ARR_LOSS)
        for i in members:
            m = pair.ref[i]
            loss_ref, grads = ot.step(pair.spec, m, i, s, pair.pool, want_grads=True)
            worst["loss"] = max(worst["loss"], abs(loss[i] - loss_ref) / max(abs(loss_ref), FLOOR))
            ge = pair.array_errors(i, binding.ARR_GRAD, grads, rms_floor=grad_floor)
            assert ge.max() <= tol_grad, (s, i, names[int(ge.argmax())], ge.max())
            worst["grad"] = max(worst["grad"], ge.max())
            cases.append(ge.max())
            we = pair.array_errors(i, binding.ARR_W32, m.theta, rms_floor=W_FLOOR, skip_key_bias=True)
            assert we.max() <= tol_w, (s, i, names[int(we.argmax())], we.max())
            worst["step"] = max(worst["step"], we.max())
            worst["s0"] = max(worst["s0"], pair.array_errors(i, binding.ARR_OPT0, m.opt["s0"], skip_key_bias=True).max())
            worst["s1"] = max(worst["s1"], pair.array_errors(i, binding.ARR_OPT1, m.opt["s1"], skip_key_bias=True).max())
            assert int(g.get(binding.ARR_T, i)[0]) == m.t
        assert worst["loss"] <= TOL_BF16 and worst["s0"] <= tol_grad and worst["s1"] <= 2 * tol_grad, (s, worst)
    worst["exact_share"] = float(np.mean(np.array(cases) <= EXACT))
    return worst


def test_transformer_reduced_steps_no_dropout():
    """Dropout 0 and smoothing 0 for one member, smoothing only for another, both for the third."""
    H = np.array([[1e-3, 0.0, 0.0], [3e-4, 0.0, 0.1], [1e-3, 0.25, 0.15]], dtype=np.float32)
    pair = TransformerPair(_reduced(), H=H)
    worst = _teacher_forced(pair, range(8), range(3))
    assert worst["exact_share"] >= 0.25, worst
    print("transformer reduced:", {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)


def test_transformer_reduced_ragged_shapes():
    """Three heads of width 8, sequence 24 and widths that leave ragged GEMM tiles."""
    wl = _reduced(P=2, vocab=72, d_model=24, heads=3, d_ff=40, n_blocks=1, seq=24, batch=3, n_eval=6)
    pair = TransformerPair(wl, H=np.array([[1e-3, 0.1, 0.05], [5e-4, 0.3, 0.0]], dtype=np.float32))
    worst = _teacher_forced(pair, range(4), range(2))
    print("transformer ragged:", {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)


@pytest.mark.parametrize("seq,batch", [(96, 2), (128, 2), (64, 2), (32, 3)])
def test_transformer_reduced_one_kernel_attention(seq, batch):
    """Heads of width 64 and sequences of 32, 96 and 128 positions take the attention kernels that keep the
    score and probability matrices on the chip (one to four query blocks); one member without
    dropout, two with."""
    wl = _reduced(P=3, vocab=64, d_model=128, heads=2, d_ff=64, n_blocks=2, seq=seq, batch=batch, n_train=16, n_eval=2 * batch)
    H = np.array([[1e-3, 0.0, 0.0], [5e-4, 0.3, 0.05], [1e-3, 0.1, 0.1]], dtype=np.float32)
    pair = TransformerPair(wl, H=H)
    # (Adam's first updates are +-lr per element whatever the gradient's size: in the zero-initialised LayerNorm
    # biases every element whose gradient is small enough to change sign within TOL_GRAD_SMALL is off by 2 lr,
    # so the updated weights are only held to the gradients' bound here, which is twice that of the smaller
    # networks above: with 64 to 256 rows per batch one differently rounded activation moves the second block's
    # feed-forward gradients by up to 5 %, and the kernels that compute attention in several launches give the
    # same distances at these shapes)
    worst = _teacher_forced(pair, range(3), range(3), tol_grad=2 * TOL_GRAD_SMALL, tol_w=2 * TOL_GRAD_SMALL)
    pair.gpu.eval(pair.d_eval)
    sc, sc_ref = pair.gpu.get(binding.ARR_SCORE), pair.eval_ref()
    worst["score"] = float(np.max(np.abs(sc - sc_ref) / np.abs(sc_ref)))
    assert worst["score"] <= TOL_BF16, (sc, sc_ref)
    print("transformer one-kernel attention, seq %d:" % seq, {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)


def test_transformer_reduced_weight_gradient_in_parts():
    """4096 rows per member and a 256 x 256 output projection: the weight gradients of the small matrices are formed
    in four pieces of the contraction and added up (here the attention projections and, with d_ff = 256, the
    feed-forward matrices too)."""
    wl = _reduced(P=2, vocab=64, d_model=256, heads=4, d_ff=256, n_blocks=1, seq=128, batch=32, n_train=64, n_eval=32)
    pair = TransformerPair(wl, H=np.array([[1e-3, 0.1, 0.05], [5e-4, 0.0, 0.0]], dtype=np.float32))
    worst = _teacher_forced(pair, range(2), range(2), tol_grad=2 * TOL_GRAD_SMALL, tol_w=2 * TOL_GRAD_SMALL)
    print("transformer weight gradient in parts:", {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)


def test_transformer_free_running_eval_and_exploit():
    pair = TransformerPair(_reduced(P=4))
    g, P = pair.gpu, 4
    worst = dict(w=0.0, loss=0.0, score=0.0)
    rnd = 0
    for s in range(12):
        g.step(pair.d_pool, s)
        loss_ref = pair.step_ref(s)
        loss = g.get(binding.ARR_LOSS)
        worst["loss"] = max(worst["loss"], float(np.max(np.abs(loss - loss_ref) / np.maximum(np.abs(loss_ref), FLOOR))))
        for i in range(P):
            worst["w"] = max(worst["w"], pair.array_errors(i, binding.ARR_W32, pair.ref[i].theta, rms_floor=W_FLOOR, skip_key_bias=True).max())
        assert worst["w"] <= TOL_BF16 and worst["loss"] <= TOL_BF16, (s, worst)
        if (s + 1) % 4 == 0:
            g.eval(pair.d_eval)
            sc = g.get(binding.ARR_SCORE)
            sc_ref = pair.eval_ref()
            worst["score"] = max(worst["score"], float(np.max(np.abs(sc - sc_ref) / np.abs(sc_ref))))
            assert worst["score"] <= TOL_BF16, (s, sc, sc_ref)
            g.exploit_explore(rnd)
            order, donor = pair.exploit_ref(rnd, sc)
            assert list(g.get(binding.ARR_ORDER)) == order and np.array_equal(g.get(binding.ARR_DONOR), donor)
            Hg = g.get(binding.ARR_HYPER)
            assert Hg.tobytes() == np.stack([pair.ref[i].h for i in range(P)]).tobytes()
            assert np.all(Hg[:, 1] <= 0.9) and np.all(Hg[:, 2] <= 0.9)
            for i in range(P):                                        # copied weights are the donor's, bit for bit
                if donor[i] >= 0:
                    assert g.get(binding.ARR_W32, i).tobytes() == g.get(binding.ARR_W32, int(donor[i])).tobytes()
                pair.sync_ref_from_gpu(i)
            rnd += 1
    print("transformer free-running:", {k: float("%.3g" % v) for k, v in worst.items()}, flush=True)


def test_transformer_dropout_mask_rate_and_eval_is_deterministic():
    """Eval ignores dropout and smoothing: the score does not change with either hyperparameter."""
    pair = TransformerPair(_reduced(P=2), H=np.array([[1e-3, 0.0, 0.0], [1e-3, 0.0, 0.0]], dtype=np.float32))
    g = pair.gpu
    g.eval(pair.d_eval)
    a = g.get(binding.ARR_SCORE).copy()
    assert a[0] != a[1] and np.all(a < -1.0)
    g.set(binding.ARR_HYPER, np.array([[1e-3, 0.5, 0.3], [1e-3, 0.2, 0.1]], dtype=np.float32))
    g.eval(pair.d_eval)
    assert g.get(binding.ARR_SCORE).tobytes() == a.tobytes()
    assert np.all(g.get(binding.ARR_T) == 0)


def test_transformer_full_size_sampled_member():
    """P = 16, 4 blocks, d_model 512, 8 heads, FFN 2048, 128 positions, vocabulary 8192, 32 sequences:
    after three steps of the whole population one member is followed by the oracle through one
    teacher-forced step.

    Loss, updated weights and optimiser moments meet the bf16 tolerance.  The gradient cannot be held
    to it array by array at this depth: stored bf16 values that round the other way under fp32
    accumulation (a few in 10^4 per tensor) spread through attention and the residual stream, and
    where a feed-forward pre-activation changes sign the ReLU gate of that element flips, a 100 %
    error on it; a share m of flipped gates moves the gradients behind them by about sqrt(2 m)
    (measured: m = 7e-5 in the first block to 7e-4 in the last, 1-4 %).  That is a property of the
    function, so the bar per array is set by the function itself: what switching the oracle from
    exact to bf16 storage moves that same gradient (the GPU must be no farther from the bf16 oracle
    than exact arithmetic is), and never above TOL_GRAD_SMALL; the gradient as one vector within 2 %."""
    from oracle import transformer as ot
    wl = workloads.TRANSFORMER
    H0 = workloads.initial_hypers(wl, 6)
    i = int(np.argmax(H0[:, 1]))                                      # the member with the highest dropout rate
    pair = TransformerPair(wl, ref_members=[i])
    g = pair.gpu
    for s in range(3):
        g.step(pair.d_pool, s)
    assert np.all(np.isfinite(g.get(binding.ARR_LOSS)))
    s = 3
    pair.sync_ref_from_gpu(i)
    m = pair.ref[i]
    exact_spec = ot.TransformerSpec(wl.vocab, wl.d_model, wl.heads, wl.d_ff, wl.n_blocks, wl.seq, wl.batch, pair.seed,
                                    roles=wl.roles, bf16_storage=False)
    twin = ot.new_member(exact_spec, [a.copy() for a in m.theta], m.h.copy(), i)
    _, grads_exact = ot.step(exact_spec, twin, i, s, pair.pool, want_grads=True)
    g.step(pair.d_pool, s)
    loss_ref, grads = ot.step(pair.spec, m, i, s, pair.pool, want_grads=True)
    names = [n for n, _ in pair.spec.param_shapes()]
    loss_err = abs(g.get(binding.ARR_LOSS)[i] - loss_ref) / max(abs(loss_ref), FLOOR)
    ge = pair.array_errors(i, binding.ARR_GRAD, grads)
    storage = np.array([np.linalg.norm(a - b) / np.linalg.norm(a) for a, b in zip(grads, grads_exact)])
    bar = np.minimum(np.maximum(TOL_BF16, storage), TOL_GRAD_SMALL)
    worst = int(np.argmax(ge / bar))
    assert np.all(ge <= bar), (names[worst], ge[worst], bar[worst])
    flat = lambda arrs: np.concatenate([a.ravel() for a in arrs])
    whole = np.linalg.norm(flat(pair.gpu_arrays(i, binding.ARR_GRAD)) - flat(grads)) / np.linalg.norm(flat(grads))
    we = pair.array_errors(i, binding.ARR_W32, m.theta, rms_floor=W_FLOOR, skip_key_bias=True).max()
    s0 = pair.array_errors(i, binding.ARR_OPT0, m.opt["s0"], skip_key_bias=True).max()
    s1 = pair.array_errors(i, binding.ARR_OPT1, m.opt["s1"], skip_key_bias=True).max()
    # the moment estimates are averages of gradients (and of their squares) and share the gradients' bar
    assert loss_err <= TOL_BF16 and we <= TOL_BF16 and whole <= 2 * TOL_BF16 and s0 <= TOL_GRAD_SMALL and s1 <= TOL_GRAD_SMALL, (loss_err, we, whole, s0, s1)
    assert int(g.get(binding.ARR_T, i)[0]) == m.t == 4
    # score of the sampled member over all 256 held-out sequences, from the GPU's current weights
    pair.sync_ref_from_gpu(i)
    g.eval(pair.d_eval)
    sc = g.get(binding.ARR_SCORE)
    sc_ref = pair.eval_ref()[0]
    assert np.all(np.isfinite(sc)) and np.all(sc < -1.0) and abs(sc[i] - sc_ref) <= TOL_BF16 * abs(sc_ref), (sc[i], sc_ref)
    print("transformer full size: score %.6g ref %.6g" % (sc[i], sc_ref))
    print("transformer full size: loss %.2e  W %.2e  s0 %.2e  s1 %.2e  gradient: whole %.2e, worst array %.2e (%s; bf16 storage moves it %.2e)"
          % (loss_err, we, s0, s1, whole, ge[worst], names[worst], storage[worst]), flush=True)
