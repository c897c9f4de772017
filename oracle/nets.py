"""Dense networks in float64: forward, loss, backward (oracle side).

`step` in the paper (Section 3, Eq. 2) is one gradient-descent update of a
member's weights theta given its hyperparameters h; this module supplies the
gradient of the training objective for the fully connected workloads.  A
network is a list of (W, b) pairs with W of shape (fan_in, fan_out); a layer
computes a @ W + b and every layer but the last is followed by the activation.
Nothing here is blocked, fused or reordered: each function is the textbook
definition written out.
"""
import numpy as np
from scipy.special import erf

ACT_NONE, ACT_RELU, ACT_GELU, ACT_LEAKY_RELU, ACT_TANH = 0, 1, 2, 3, 4
LEAKY_SLOPE = 0.2


def act(z, kind):
    if kind == ACT_NONE:
        return z
    if kind == ACT_RELU:
        return np.where(z > 0.0, z, 0.0)
    if kind == ACT_GELU:                       # exact form: z * Phi(z)
        return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))
    if kind == ACT_LEAKY_RELU:
        return np.where(z > 0.0, z, LEAKY_SLOPE * z)
    if kind == ACT_TANH:
        return np.tanh(z)
    raise ValueError(kind)


def act_grad(z, kind):
    """d act(z) / dz, elementwise."""
    if kind == ACT_NONE:
        return np.ones_like(z)
    if kind == ACT_RELU:
        return np.where(z > 0.0, 1.0, 0.0)
    if kind == ACT_GELU:                       # Phi(z) + z * phi(z)
        return 0.5 * (1.0 + erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)
    if kind == ACT_LEAKY_RELU:
        return np.where(z > 0.0, 1.0, LEAKY_SLOPE)
    if kind == ACT_TANH:
        return 1.0 - np.tanh(z) ** 2
    raise ValueError(kind)


def round_bf16(x):
    """Nearest bfloat16 value (8 significant bits), ties to even, returned as float64.
    bfloat16 keeps 7 of float64's 52 stored mantissa bits, so the low 45 bits are
    rounded away.  (Below 2**-126, where bfloat16 goes subnormal, this keeps more
    precision than the real format; nothing here lives there.)"""
    u = np.ascontiguousarray(x, dtype=np.float64).view(np.uint64)
    lsb = (u >> np.uint64(45)) & np.uint64(1)
    u = u + np.uint64((1 << 44) - 1) + lsb
    u = u & ~np.uint64((1 << 45) - 1)
    return u.view(np.float64)


def identity(x):
    return x


def mlp_forward(params, x, hidden_act, out_act=ACT_NONE, q=identity):
    """Returns (output, cache).  cache = (inputs to each layer, pre-activations).

    q is the storage rounding of mixed-precision training (identity for full
    precision, round_bf16 for "bf16 compute with fp32 master weights"): the two
    operands of every dense contraction -- layer inputs and weights -- and every
    hidden tensor kept for the backward pass are rounded by q; biases, the
    output layer's result and all sums are not."""
    a = q(np.asarray(x, dtype=np.float64))
    ins, zs = [], []
    L = len(params)
    for l, (W, b) in enumerate(params):
        ins.append(a)
        z = a @ q(W) + b
        if l < L - 1:
            zs.append(q(z))
            a = q(act(z, hidden_act))
        else:
            # the last pre-activation is kept for the backward pass only when an output
            # non-linearity follows (a generator's tanh); plain logits are not stored
            zs.append(q(z) if out_act != ACT_NONE else z)
            a = act(z, out_act)
    return a, (ins, zs)


def mlp_backward(params, cache, d_out, hidden_act, out_act=ACT_NONE, q=identity):
    """Given dLoss/d(output), returns ([(dW, db), ...], dLoss/d(input)).
    With a storage rounding q, the gradient with respect to every layer's
    pre-activation (the logits included) is rounded before it enters the
    contractions that produce weight, bias and input gradients."""
    ins, zs = cache
    L = len(params)
    grads = [None] * L
    da = d_out
    for l in range(L - 1, -1, -1):
        W, _ = params[l]
        dz = q(da * act_grad(zs[l], hidden_act if l < L - 1 else out_act))
        grads[l] = (ins[l].T @ dz, dz.sum(axis=0))
        da = dz @ q(W).T
    return grads, da


def log_softmax(logits):
    m = logits.max(axis=-1, keepdims=True)
    s = logits - m
    return s - np.log(np.exp(s).sum(axis=-1, keepdims=True))


def softmax_xent(logits, labels, smoothing=0.0):
    """Mean over rows of the cross-entropy between the (label-smoothed) target
    distribution and softmax(logits).  Returns (loss, dLoss/dlogits).
    Target: (1 - smoothing) on the label plus smoothing / C on every class."""
    n, C = logits.shape
    lsm = log_softmax(logits)
    q = np.full((n, C), smoothing / C)
    q[np.arange(n), labels] += 1.0 - smoothing
    loss = -(q * lsm).sum() / n
    dlogits = (np.exp(lsm) - q) / n
    return loss, dlogits


def softplus(x):
    """log(1 + e^x), evaluated without overflow."""
    return np.maximum(x, 0.0) + np.log1p(np.exp(-np.abs(x)))


def sigmoid(x):
    return np.where(x >= 0, 1.0 / (1.0 + np.exp(-np.abs(x))), np.exp(-np.abs(x)) / (1.0 + np.exp(-np.abs(x))))


def logistic_loss(logits, targets):
    """Mean binary cross-entropy of sigmoid(logits) against targets in {0, 1}:
    -[t log s + (1 - t) log(1 - s)] = softplus(-l) for t = 1, softplus(l) for t = 0.
    Returns (loss, dLoss/dlogits); logits has shape (n, 1) or (n,)."""
    l = np.asarray(logits, dtype=np.float64).reshape(-1)
    t = np.asarray(targets, dtype=np.float64).reshape(-1)
    loss = np.mean(np.where(t > 0.5, softplus(-l), softplus(l)))
    d = (sigmoid(l) - t) / len(l)
    return loss, d.reshape(np.shape(logits))


def classifier_loss_and_grads(params, x, labels, hidden_act, q=identity):
    """Training objective of the classifier workloads: mean softmax cross-entropy."""
    logits, cache = mlp_forward(params, x, hidden_act, q=q)
    loss, dlogits = softmax_xent(logits, labels)
    grads, _ = mlp_backward(params, cache, dlogits, hidden_act, q=q)
    return loss, grads


def classifier_eval_loss(params, x, labels, hidden_act, q=identity):
    logits, _ = mlp_forward(params, x, hidden_act, q=q)
    loss, _ = softmax_xent(logits, labels)
    return loss
