"""`step` and `eval` for the language-model workload (oracle side).

The paper's supervised experiment (Section 4.2.1) trains Transformer networks
with Adam, lets PBT adapt the learning rate and several dropout rates, and
scores members with a metric that is not the training loss.  This synthetic
stand-in keeps that structure with a decoder-only transformer on synthetic
token sequences:

  network  token + learned position embeddings; n_layers pre-LayerNorm blocks
               h <- h + drop(attn(LN1(h)))      causal multi-head self-attention
               h <- h + drop(W2 drop(relu(W1 LN2(h))))
           a final LayerNorm and an untied linear head over the vocabulary.
           One dropout rate p is applied at four places per block: attention
           probabilities, attention output, feed-forward hidden, feed-forward
           output.  LayerNorm eps = 1e-5.
  step     B sequences drawn from a pool (Philox domain 1, one draw per
           sequence); loss = mean over the B*S positions of the label-smoothed
           cross-entropy of the next token (target = (1-e) onehot + e/V);
           one Adam update with the member's learning rate; p and e are the
           member's second and third hyperparameters.
  eval     minus the perplexity exp(mean cross-entropy) of the next token on
           held-out sequences, without dropout or smoothing.

Dropout masks come from Philox: element i of site s keeps its value iff word
i % 4 of counter (step, member, DOMAIN_DROPOUT + s, i // 4) is >= floor(p * 2^32)
(capped at 2^32 - 1), p the float32 rate widened exactly; kept values are scaled
by the float32 number nearest to 1/(1-p) (the factor is a device-resident
float32 like the rate it comes from; naming its precision matters because
bf16 values times a factor like 10/7 or 4/3 often land within 1e-8 of the
midpoint between two bf16 values, where the last bits of the factor decide
the rounding).  Sites are numbered 4*layer + {0: attention probabilities [B][H][S][S],
1: attention output [B*S][d], 2: feed-forward hidden [B*S][f], 3: feed-forward
output [B*S][d]}.

Mixed precision: with bf16 storage every tensor that is written to memory
between two operations (GEMM results, LayerNorm / softmax / dropout / residual
outputs, and their gradients) is rounded by q; logits, losses, LayerNorm
statistics, biases, gains and the optimiser stay in full precision, and GEMMs
read q(W).
"""
import numpy as np

from . import nets, optim, philox, pbt

ROLE_LR, ROLE_DROPOUT, ROLE_LABEL_SMOOTH = 0, 6, 7
LN_EPS = 1e-5


class TransformerSpec:
    def __init__(self, vocab, d_model, n_heads, d_ff, n_layers, seq, batch, seed,
                 roles=(ROLE_LR, ROLE_DROPOUT, ROLE_LABEL_SMOOTH), beta1=0.9, beta2=0.999, eps=1e-8, bf16_storage=False):
        assert d_model % n_heads == 0
        self.V, self.d, self.H, self.f, self.L, self.S, self.B = vocab, d_model, n_heads, d_ff, n_layers, seq, batch
        self.seed, self.roles = seed, list(roles)
        self.beta1, self.beta2, self.eps = beta1, beta2, eps
        self.q = nets.round_bf16 if bf16_storage else nets.identity

    def param_shapes(self):
        """Names and shapes of the parameter arrays, in the order of the flat parameter vector."""
        d, f, V, S = self.d, self.f, self.V, self.S
        out = [("tok_emb", (V, d)), ("pos_emb", (S, d))]
        for l in range(self.L):
            out += [("ln1_g%d" % l, (d,)), ("ln1_b%d" % l, (d,)), ("wqkv%d" % l, (d, 3 * d)), ("bqkv%d" % l, (3 * d,)),
                    ("wo%d" % l, (d, d)), ("bo%d" % l, (d,)), ("ln2_g%d" % l, (d,)), ("ln2_b%d" % l, (d,)),
                    ("w1%d" % l, (d, f)), ("b1%d" % l, (f,)), ("w2%d" % l, (f, d)), ("b2%d" % l, (d,))]
        out += [("lnf_g", (d,)), ("lnf_b", (d,)), ("whead", (d, V)), ("bhead", (V,))]
        return out


def init_arrays(spec, seed, member, starts):
    """Initial parameter arrays of one member (Figure 1c: random weight initialisations): token and
    position tables and all matrices uniform in +-1/sqrt(fan_in) (fan_in = d_model for the tables),
    LayerNorm gains 1, every bias 0; starts[j] = position of array j in the member's flat vector."""
    segs = []
    for (name, shape), start in zip(spec.param_shapes(), starts):
        if name in ("tok_emb", "pos_emb"):
            segs.append((start, shape, spec.d, 0.0))
        elif len(shape) == 2:
            segs.append((start, shape, shape[0], 0.0))
        else:
            segs.append((start, shape, 0, 1.0 if "_g" in name else 0.0))
    return pbt.init_segments(seed, member, segs)


def new_member(spec, arrays, h, index):
    flat = [np.array(a, dtype=np.float64) for a in arrays]
    assert [a.shape for a in flat] == [s for _, s in spec.param_shapes()]
    return pbt.Member(flat, h, {"s0": [np.zeros_like(a) for a in flat], "s1": [np.zeros_like(a) for a in flat]}, index)


def params_of(spec, m):
    return {name: a for (name, _), a in zip(spec.param_shapes(), m.theta)}


def dropout_keep(seed, step, member, site, n, p32):
    """Boolean keep mask of n elements for rate p32 (a float32 value)."""
    thr = min(int(np.floor(np.float64(p32) * 4294967296.0)), 4294967295)
    # element e takes word e % 4 of counter e // 4: the words of counters 0, 1, 2, ... laid end to end
    w = philox.words(seed, step, member, philox.DOMAIN_DROPOUT + site, np.arange((n + 3) // 4))
    return w.reshape(-1)[:n].astype(np.uint64) >= np.uint64(thr)


def layernorm(x, g, b):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xhat = (x - mu) * rstd
    return xhat * g + b, (xhat, rstd)


def layernorm_backward(dy, g, cache):
    xhat, rstd = cache
    dyg = dy * g
    dx = rstd * (dyg - dyg.mean(axis=-1, keepdims=True) - xhat * (dyg * xhat).mean(axis=-1, keepdims=True))
    return dx, (dy * xhat).sum(axis=0), dy.sum(axis=0)


def causal_softmax(s):
    """s [..., S, S]; position t attends to positions <= t."""
    S = s.shape[-1]
    mask = np.tril(np.ones((S, S), dtype=bool))
    s = np.where(mask, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


class _Drop:
    """Dropout of one step: masks by site (rate 0 or eval: everything kept, scale 1)."""

    def __init__(self, spec, step, member, p32, active):
        self.spec, self.step, self.member = spec, step, member
        self.p32 = np.float32(p32)
        self.active = active and float(p32) > 0.0
        self.scale = float(np.float32(1.0 / (1.0 - float(self.p32)))) if self.active else 1.0

    def mask(self, site, shape):
        if not self.active:
            return np.ones(shape)
        keep = dropout_keep(self.spec.seed, self.step, self.member, site, int(np.prod(shape)), self.p32)
        return keep.reshape(shape) * self.scale


def forward(spec, P, tokens, drop):
    """tokens [B][S] ints.  Returns (logits [B*S][V], cache)."""
    q = spec.q
    B, S = tokens.shape
    d, H = spec.d, spec.H
    dh = d // H
    n = B * S
    c = {"tokens": tokens}
    h = q(q(P["tok_emb"])[tokens] + q(P["pos_emb"])[None, :S, :]).reshape(n, d)
    c["layers"] = []
    for l in range(spec.L):
        lc = {"h_in": h}
        y, lc["ln1"] = layernorm(h, P["ln1_g%d" % l], P["ln1_b%d" % l])
        u = q(y)
        qkv = q(u @ q(P["wqkv%d" % l]) + P["bqkv%d" % l])
        heads = qkv.reshape(B, S, 3, H, dh).transpose(2, 0, 3, 1, 4)          # [3][B][H][S][dh]
        qh, kh, vh = heads[0], heads[1], heads[2]
        s = q(qh @ kh.transpose(0, 1, 3, 2))                                  # raw scores, stored
        p = causal_softmax(s * (1.0 / np.sqrt(dh)))
        m0 = drop.mask(4 * l + 0, p.shape)
        pq, pd = q(p), q(p * m0)                                              # probabilities kept for backward; dropped ones feed P V
        o = q(pd @ vh).transpose(0, 2, 1, 3).reshape(n, d)
        a = q(o @ q(P["wo%d" % l]) + P["bo%d" % l])
        m1 = drop.mask(4 * l + 1, a.shape)
        h = q(h + a * m1)
        lc.update(u=u, qh=qh, kh=kh, vh=vh, pq=pq, pd=pd, m0=m0, o=o, m1=m1, h_mid=h)
        y, lc["ln2"] = layernorm(h, P["ln2_g%d" % l], P["ln2_b%d" % l])
        u2 = q(y)
        f = u2 @ q(P["w1%d" % l]) + P["b1%d" % l]
        z1, r = q(f), q(np.maximum(f, 0.0))
        m2 = drop.mask(4 * l + 2, r.shape)
        fd = q(r * m2)
        g = q(fd @ q(P["w2%d" % l]) + P["b2%d" % l])
        m3 = drop.mask(4 * l + 3, g.shape)
        h = q(h + g * m3)
        lc.update(u2=u2, z1=z1, fd=fd, m2=m2, m3=m3)
        c["layers"].append(lc)
    y, c["lnf"] = layernorm(h, P["lnf_g"], P["lnf_b"])
    uf = q(y)
    c["uf"] = uf
    logits = uf @ q(P["whead"]) + P["bhead"]
    return logits, c


def backward(spec, P, cache, dlogits):
    """Gradients of all parameter arrays (dict by name) given dLoss/dlogits [B*S][V]."""
    q = spec.q
    tokens = cache["tokens"]
    B, S = tokens.shape
    d, H = spec.d, spec.H
    dh = d // H
    n = B * S
    G = {}
    dl = q(dlogits)
    G["whead"], G["bhead"] = cache["uf"].T @ dl, dl.sum(axis=0)
    du = q(dl @ q(P["whead"]).T)
    dx, G["lnf_g"], G["lnf_b"] = layernorm_backward(du, P["lnf_g"], cache["lnf"])
    dhid = q(dx)
    for l in range(spec.L - 1, -1, -1):
        lc = cache["layers"][l]
        # feed-forward branch
        dg = q(dhid * lc["m3"])
        G["w2%d" % l], G["b2%d" % l] = lc["fd"].T @ dg, dg.sum(axis=0)
        dfd = q(dg @ q(P["w2%d" % l]).T)
        dz1 = q(dfd * lc["m2"] * (lc["z1"] > 0.0))
        G["w1%d" % l], G["b1%d" % l] = lc["u2"].T @ dz1, dz1.sum(axis=0)
        du2 = q(dz1 @ q(P["w1%d" % l]).T)
        dx, G["ln2_g%d" % l], G["ln2_b%d" % l] = layernorm_backward(du2, P["ln2_g%d" % l], lc["ln2"])
        dhid = q(dhid + dx)
        # attention branch
        da = q(dhid * lc["m1"])
        G["wo%d" % l], G["bo%d" % l] = lc["o"].T @ da, da.sum(axis=0)
        do = q(da @ q(P["wo%d" % l]).T).reshape(B, S, H, dh).transpose(0, 2, 1, 3)      # [B][H][S][dh]
        dv = q(lc["pd"].transpose(0, 1, 3, 2) @ do)
        dpd = q(do @ lc["vh"].transpose(0, 1, 3, 2))
        dp = dpd * lc["m0"]
        ds = q(lc["pq"] * (dp - (dp * lc["pq"]).sum(axis=-1, keepdims=True)) * (1.0 / np.sqrt(dh)))
        dq = q(ds @ lc["kh"])
        dk = q(ds.transpose(0, 1, 3, 2) @ lc["qh"])
        dqkv = np.stack([dq, dk, dv]).transpose(1, 3, 0, 2, 4).reshape(n, 3 * d)       # [B][S][3][H][dh]
        G["wqkv%d" % l], G["bqkv%d" % l] = lc["u"].T @ dqkv, dqkv.sum(axis=0)
        duu = q(dqkv @ q(P["wqkv%d" % l]).T)
        dx, G["ln1_g%d" % l], G["ln1_b%d" % l] = layernorm_backward(duu, P["ln1_g%d" % l], lc["ln1"])
        dhid = q(dhid + dx)
    dh0 = dhid.reshape(B, S, d)
    G["pos_emb"] = np.zeros_like(P["pos_emb"])
    G["pos_emb"][:S] = dh0.sum(axis=0)
    G["tok_emb"] = np.zeros_like(P["tok_emb"])
    np.add.at(G["tok_emb"], tokens.reshape(-1), dh0.reshape(n, d))
    return G


def loss_and_grads(spec, m, seqs, step, member, train=True):
    """seqs [B][S+1] ints: inputs are positions 0..S-1, targets positions 1..S."""
    P = params_of(spec, m)
    p32 = m.h[spec.roles.index(ROLE_DROPOUT)] if ROLE_DROPOUT in spec.roles else np.float32(0)
    ls = float(m.h[spec.roles.index(ROLE_LABEL_SMOOTH)]) if ROLE_LABEL_SMOOTH in spec.roles else 0.0
    drop = _Drop(spec, step, member, p32, train)
    tokens, targets = seqs[:, :-1], seqs[:, 1:].reshape(-1)
    logits, cache = forward(spec, P, tokens, drop)
    loss, dlogits = nets.softmax_xent(logits, targets, ls if train else 0.0)
    if not train:
        return loss, None
    G = backward(spec, P, cache, dlogits)
    return loss, [G[name] for name, _ in spec.param_shapes()]


def step(spec, m, i, s, pool, want_grads=False):
    """One update of member i at step s; returns the loss (and the gradients it used, if asked)."""
    idx = philox.bounded(philox.words(spec.seed, s, i, philox.DOMAIN_BATCH, np.arange(spec.B))[..., 0], len(pool))
    loss, grads = loss_and_grads(spec, m, pool[idx], s, i)
    lr = m.h[spec.roles.index(ROLE_LR)]
    m.t += 1
    for j, g in enumerate(grads):
        m.theta[j], m.opt["s0"][j], m.opt["s1"][j] = optim.adam(
            m.theta[j], g, m.opt["s0"][j], m.opt["s1"][j], m.t, lr, spec.beta1, spec.beta2, spec.eps, 0.0)
    return (loss, grads) if want_grads else loss


def evaluate(spec, m, eval_seqs, chunk=64):
    """`eval`: minus exp(mean next-token cross-entropy) over the held-out sequences."""
    total = 0.0
    for r0 in range(0, len(eval_seqs), chunk):
        part = eval_seqs[r0:r0 + chunk]
        loss, _ = loss_and_grads(spec, m, part, 0, 0, train=False)
        total += loss * part.shape[0]
    return -np.exp(total / len(eval_seqs))
