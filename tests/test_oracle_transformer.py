"""Pins for the oracle's transformer workload: finite differences through the whole network (with and
without dropout), LayerNorm and attention closed forms, causality, the dropout mask definition, and
the perplexity / label-smoothing closed forms at a zero head."""
import math
import numpy as np
import torch

from oracle import transformer as tf, philox, nets


def _spec(bf16=False, L=2):
    return tf.TransformerSpec(vocab=11, d_model=8, n_heads=2, d_ff=12, n_layers=L, seq=5, batch=2, seed=3, bf16_storage=bf16)


def _member(spec, rng, h=(1e-3, 0.0, 0.0)):
    arrays = []
    for name, shape in spec.param_shapes():
        if name.startswith("ln") and "_g" in name:
            arrays.append(1.0 + 0.1 * rng.standard_normal(shape))
        else:
            arrays.append(0.4 * rng.standard_normal(shape))
    return tf.new_member(spec, arrays, h, 0)


def _fd(spec, m, seqs, step, tol=2e-6):
    loss, grads = tf.loss_and_grads(spec, m, seqs, step, 0)
    e = 1e-6
    rng = np.random.default_rng(0)
    for arr, g, (name, _) in zip(m.theta, grads, spec.param_shapes()):
        idxs = list(np.ndindex(*arr.shape))
        for k in rng.choice(len(idxs), size=min(6, len(idxs)), replace=False):
            idx = idxs[k]
            old = arr[idx]
            arr[idx] = old + e
            lp = tf.loss_and_grads(spec, m, seqs, step, 0)[0]
            arr[idx] = old - e
            lm = tf.loss_and_grads(spec, m, seqs, step, 0)[0]
            arr[idx] = old
            assert abs((lp - lm) / (2 * e) - g[idx]) <= tol * max(1.0, abs(g[idx])), (name, idx, (lp - lm) / (2 * e), g[idx])


def test_gradients_fd_no_dropout():
    spec = _spec()
    rng = np.random.default_rng(1)
    m = _member(spec, rng, h=(1e-3, 0.0, 0.1))
    seqs = rng.integers(0, 11, (2, 6))
    _fd(spec, m, seqs, 0)


def test_gradients_fd_with_dropout_masks():
    spec = _spec()
    rng = np.random.default_rng(2)
    m = _member(spec, rng, h=(1e-3, 0.3, 0.0))
    seqs = rng.integers(0, 11, (2, 6))
    l_a = tf.loss_and_grads(spec, m, seqs, 4, 0)[0]
    l_b = tf.loss_and_grads(spec, m, seqs, 5, 0)[0]
    assert l_a != l_b                                         # another step, another mask
    _fd(spec, m, seqs, 4)


def test_layernorm_forward_backward():
    rng = np.random.default_rng(3)
    x, g, b = rng.standard_normal((4, 8)) * 3 + 1, rng.standard_normal(8), rng.standard_normal(8)
    y, cache = tf.layernorm(x, g, b)
    xhat = (y - b) / g
    assert np.allclose(xhat.mean(axis=1), 0, atol=1e-12) and np.allclose((xhat ** 2).mean(axis=1), 1, atol=1e-4)
    ref = torch.nn.functional.layer_norm(torch.tensor(x), (8,), torch.tensor(g), torch.tensor(b), eps=1e-5)
    assert np.allclose(y, ref.numpy(), atol=1e-12)
    w = rng.standard_normal((4, 8))
    dx, dg, db = tf.layernorm_backward(w, g, cache)
    xt, gt, bt = torch.tensor(x, requires_grad=True), torch.tensor(g, requires_grad=True), torch.tensor(b, requires_grad=True)
    (torch.nn.functional.layer_norm(xt, (8,), gt, bt, eps=1e-5) * torch.tensor(w)).sum().backward()
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-12) and np.allclose(dg, gt.grad.numpy(), atol=1e-12)
    assert np.allclose(db, bt.grad.numpy(), atol=1e-12)


def test_causal_softmax_rows_and_mask():
    rng = np.random.default_rng(4)
    p = tf.causal_softmax(rng.standard_normal((2, 3, 5, 5)))
    assert np.allclose(p.sum(axis=-1), 1.0) and np.all(np.triu(p[0, 0], 1) == 0.0)
    assert p[1, 2, 0, 0] == 1.0                               # the first position can only see itself


def test_causality_of_the_whole_network():
    spec = _spec()
    rng = np.random.default_rng(5)
    m = _member(spec, rng)
    P = tf.params_of(spec, m)
    tok = rng.integers(0, 11, (2, 5))
    drop = tf._Drop(spec, 0, 0, 0.0, False)
    a, _ = tf.forward(spec, P, tok, drop)
    tok2 = tok.copy()
    tok2[:, 3] = (tok2[:, 3] + 1) % 11                        # change position 3
    b, _ = tf.forward(spec, P, tok2, drop)
    a, b = a.reshape(2, 5, 11), b.reshape(2, 5, 11)
    assert np.array_equal(a[:, :3], b[:, :3]) and not np.allclose(a[:, 3:], b[:, 3:])


def test_attention_matches_library():
    spec = _spec(L=1)
    rng = np.random.default_rng(6)
    q, k, v = (rng.standard_normal((2, 2, 5, 4)) for _ in range(3))
    ours = tf.causal_softmax(q @ k.transpose(0, 1, 3, 2) / math.sqrt(4)) @ v
    ref = torch.nn.functional.scaled_dot_product_attention(torch.tensor(q), torch.tensor(k), torch.tensor(v), is_causal=True)
    assert np.allclose(ours, ref.numpy(), atol=1e-12)


def test_zero_head_closed_forms():
    # with a zero output layer every next-token distribution is uniform: loss = ln V for any
    # label smoothing, perplexity = V exactly
    spec = _spec()
    rng = np.random.default_rng(7)
    m = _member(spec, rng, h=(1e-3, 0.2, 0.15))
    names = [n for n, _ in spec.param_shapes()]
    m.theta[names.index("whead")][:] = 0.0
    m.theta[names.index("bhead")][:] = 0.0
    seqs = rng.integers(0, 11, (4, 6))
    assert abs(tf.loss_and_grads(spec, m, seqs, 0, 0)[0] - math.log(11)) < 1e-12
    assert abs(tf.evaluate(spec, m, seqs, chunk=3) + 11.0) < 1e-10


def test_dropout_mask_definition_and_rate():
    p32 = np.float32(0.3)
    keep = tf.dropout_keep(9, 2, 1, 5, 40000, p32)
    assert abs(keep.mean() - 0.7) < 0.01
    thr = int(math.floor(float(p32) * 2 ** 32))
    for i in (0, 1, 7, 1234):
        w = philox.philox4x32_10([2, 1, philox.DOMAIN_DROPOUT + 5, i // 4], [9, 0])
        assert bool(keep[i]) == (int(w[i % 4]) >= thr)
    assert tf.dropout_keep(9, 2, 1, 5, 100, np.float32(0.0)).all()
    d = tf._Drop(_spec(), 2, 1, p32, True)
    mk = d.mask(5, (100, 4))
    kept = set(np.unique(mk)) - {0.0}
    assert len(kept) == 1
    scale = kept.pop()
    assert scale == float(np.float32(scale)) and abs(scale * (1.0 - float(p32)) - 1.0) < 6e-8    # the float32 nearest 1/(1-p)
    assert abs(mk.mean() - 1.0) < 0.15                                                          # inverted dropout keeps the mean


def test_step_trains_and_bf16_storage_is_close():
    spec, spec16 = _spec(), _spec(True)
    rng = np.random.default_rng(8)
    pool = rng.integers(0, 11, (16, 6))
    pool[:, 1:] = (pool[:, :-1] * 3 + 1) % 11                 # deterministic successor: learnable
    m = _member(spec, np.random.default_rng(9), h=(3e-2, 0.0, 0.0))
    first = tf.step(spec, m, 0, 0, pool)
    for s in range(1, 150):
        last = tf.step(spec, m, 0, s, pool)
    assert last < 0.6 * first and m.t == 150
    a, b = _member(spec, np.random.default_rng(10)), _member(spec16, np.random.default_rng(10))
    la, ga = tf.loss_and_grads(spec, a, pool[:2], 0, 0)
    lb, gb = tf.loss_and_grads(spec16, b, pool[:2], 0, 0)
    assert 0 < abs(la - lb) < 3e-2 * la
    names = [n for n, _ in spec.param_shapes()]
    for nm in ("whead", "w10", "wqkv0", "tok_emb"):
        j = names.index(nm)
        assert np.linalg.norm(ga[j] - gb[j]) < 0.35 * np.linalg.norm(ga[j])   # many rounding points, width-8 layers


def test_init_arrays_rule():
    spec = _spec()
    starts, pos = [], 0
    for _, shape in spec.param_shapes():
        starts.append(pos)
        pos += -(-int(np.prod(shape)) // 64) * 64
    arrays = tf.init_arrays(spec, 5, 1, starts)
    for (name, shape), a in zip(spec.param_shapes(), arrays):
        assert a.shape == shape and a.dtype == np.float32
        if len(shape) == 2:
            fan = spec.d if name.endswith("_emb") else shape[0]
            assert np.all(np.abs(a) < 1 / math.sqrt(fan)) and a.std() > 0.3 / math.sqrt(fan)
        else:
            assert np.all(a == (1.0 if "_g" in name else 0.0))
    again = tf.init_arrays(spec, 5, 2, starts)
    assert not np.array_equal(arrays[0], again[0])                       # members are initialised independently
