"""Parameter update (oracle; test infrastructure only).

Algorithm 1 line 11: theta <- theta - lambda * grad.  The experiments (Appendix B) use Adam;
the paper gives only the learning rate, so the usual defaults are taken (beta1 0.9,
beta2 0.999, eps 1e-8, bias correction, no weight decay).  float64.
"""
import numpy as np


def sgd(theta, grad, lr):
    return np.asarray(theta, np.float64) - float(lr) * np.asarray(grad, np.float64)


def adam(theta, grad, m, v, lr, t, b1=0.9, b2=0.999, eps=1e-8):
    """One Adam step; t is the 1-based step count.  Returns (theta, m, v)."""
    g = np.asarray(grad, np.float64)
    m = b1 * np.asarray(m, np.float64) + (1.0 - b1) * g
    v = b2 * np.asarray(v, np.float64) + (1.0 - b2) * g * g
    mhat = m / (1.0 - b1 ** t)
    vhat = v / (1.0 - b2 ** t)
    return np.asarray(theta, np.float64) - lr * mhat / (np.sqrt(vhat) + eps), m, v
