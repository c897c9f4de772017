"""`step` and `eval` for the supervised classifier workloads (oracle side).

`step` (Section 3, Eq. 2) = one mini-batch gradient update of the mean softmax
cross-entropy under the member's hyperparameters; `eval` (Section 3, Eq. 1) =
negative mean cross-entropy on a held-out set ("validation set performance",
Section 3).  Which rows member i sees at step s is not fixed by the paper; the
reading is B independent uniform draws (with replacement) from the training
set, from Philox counter (s, i, DOMAIN_BATCH, row).
"""
import numpy as np

from . import nets, optim, philox, pbt

OPT_SGD_MOMENTUM, OPT_ADAM, OPT_RMSPROP = 0, 1, 2
# hyperparameter roles (what a column of h means)
ROLE_LR, ROLE_BETA1, ROLE_WD = 0, 1, 2


class ClassifierSpec:
    def __init__(self, dims, hidden_act, optimizer, batch, roles, seed,
                 momentum=0.9, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.0, rho=0.99, rms_eps=1e-5,
                 bf16_storage=False):
        self.dims = list(dims)
        self.hidden_act = hidden_act
        self.optimizer = optimizer
        self.batch = batch
        self.roles = list(roles)
        self.seed = seed
        self.momentum, self.beta1, self.beta2, self.eps, self.wd = momentum, beta1, beta2, eps, wd
        self.rho, self.rms_eps = rho, rms_eps
        # mixed precision: contraction operands and stored hidden tensors rounded to bfloat16
        self.q = nets.round_bf16 if bf16_storage else nets.identity


def batch_rows(seed, s, i, batch, n_train):
    rows = np.arange(batch)
    x = philox.words(seed, s, i, philox.DOMAIN_BATCH, rows)[..., 0]
    return philox.bounded(x, n_train)


def new_member(spec, theta, h, index):
    """theta: list of (W, b).  Optimiser state starts at zero."""
    flat = [np.array(a, dtype=np.float64) for Wb in theta for a in Wb]
    n_state = {OPT_SGD_MOMENTUM: 1, OPT_ADAM: 2, OPT_RMSPROP: 1}[spec.optimizer]
    opt = {"s%d" % k: [np.zeros_like(a) for a in flat] for k in range(n_state)}
    return pbt.Member(flat, h, opt, index)


def params_of(member):
    th = member.theta
    return [(th[2 * l], th[2 * l + 1]) for l in range(len(th) // 2)]


def hyper(spec, member, role, default):
    return member.h[spec.roles.index(role)] if role in spec.roles else default


def apply_optimizer(spec, member, flat_grads):
    """theta <- update(theta, g, state | h) for every parameter array."""
    lr = hyper(spec, member, ROLE_LR, None)
    member.t += 1
    for j, g in enumerate(flat_grads):
        th = member.theta[j]
        if spec.optimizer == OPT_SGD_MOMENTUM:
            th, member.opt["s0"][j] = optim.sgd_momentum(th, g, member.opt["s0"][j], lr, spec.momentum)
        elif spec.optimizer == OPT_ADAM:
            b1 = hyper(spec, member, ROLE_BETA1, spec.beta1)
            wd = hyper(spec, member, ROLE_WD, spec.wd)
            th, member.opt["s0"][j], member.opt["s1"][j] = optim.adam(
                th, g, member.opt["s0"][j], member.opt["s1"][j], member.t, lr, b1, spec.beta2, spec.eps, wd)
        elif spec.optimizer == OPT_RMSPROP:
            th, member.opt["s0"][j] = optim.rmsprop(th, g, member.opt["s0"][j], lr, spec.rho, spec.rms_eps)
        else:
            raise ValueError(spec.optimizer)
        member.theta[j] = th


def step(spec, member, i, s, train_x, train_y):
    """One `step`.  Returns the mini-batch loss (before the update)."""
    rows = batch_rows(spec.seed, s, i, spec.batch, len(train_y))
    loss, grads = nets.classifier_loss_and_grads(params_of(member), train_x[rows], train_y[rows],
                                                 spec.hidden_act, spec.q)
    apply_optimizer(spec, member, [a for g in grads for a in g])
    return loss


def evaluate(spec, member, eval_x, eval_y):
    """`eval`: negative mean cross-entropy on the held-out set."""
    return -nets.classifier_eval_loss(params_of(member), eval_x, eval_y, spec.hidden_act, spec.q)
