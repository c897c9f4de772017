"""Per-member optimiser updates in float64 (oracle side).

The paper names the optimisers (SGD or RMSProp in Section 3; RMSProp for the RL
experiments, Section 4.1.1; Adam for translation and GANs, Sections 4.2.1 and
4.3.1, with beta1 = 0.5, beta2 = 0.999, eps = 1e-8 in the GAN appendix) but not
their formulas.  The readings taken here:

  SGD-momentum  v <- mu v + g ;  theta <- theta - lr v      (lr outside the buffer, so a
                                                             perturbed lr acts at once)
  Adam          m <- b1 m + (1-b1) g ; v <- b2 v + (1-b2) g^2 ; t <- t + 1
                theta <- theta - lr ( (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps) + wd theta )
                (decoupled weight decay on every parameter; b1^t uses the member's
                 current b1, which exploit/explore may have changed)
  RMSProp       s <- rho s + (1-rho) g^2 ; theta <- theta - lr g / sqrt(s + eps)

lr, b1, wd arrive as float32 hyperparameters and are widened exactly.
Each function updates one parameter array and returns the new arrays.
"""
import numpy as np


def sgd_momentum(theta, g, v, lr, mu):
    v = mu * v + g
    theta = theta - float(lr) * v
    return theta, v


def adam(theta, g, m, v, t, lr, beta1, beta2, eps, wd):
    """t is the step count AFTER this update (first update: t = 1)."""
    lr, beta1, wd = float(lr), float(beta1), float(wd)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    theta = theta - lr * (mhat / (np.sqrt(vhat) + eps) + wd * theta)
    return theta, m, v


def rmsprop(theta, g, s, lr, rho, eps):
    s = rho * s + (1.0 - rho) * g * g
    theta = theta - float(lr) * g / np.sqrt(s + eps)
    return theta, s
