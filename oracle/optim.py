"""Oracle of the model updates that consume the estimates (TEST INFRASTRUCTURE, see
agc_oracle.c): plain gradient descent (Sec. II-A, update rule) and the Adam step fed by the two
decoding tracks (Sec. V, extension to adaptive optimizers; ratio of Appendix F).  binary64 numpy.
"""
import numpy as np


def gd_update(beta, ghat, lr):
    """beta - lr * ghat."""
    return np.asarray(beta, dtype=np.float64) - float(lr) * np.asarray(ghat, dtype=np.float64)


def adam_update(beta, m1, m2, ghat, ghat2, lr, beta1, beta2, eps, t):
    """One Adam step at iteration t >= 1: the first-moment average takes the unbiased estimate
    ghat, the second-moment average the square of the variance-reduced estimate ghat2; the
    customary bias corrections 1 - beta^t and the eps in the denominator (the paper prints only
    the ratio chi_t / sqrt(nu_t)).  Returns (beta, m1, m2)."""
    beta, m1, m2 = (np.asarray(x, dtype=np.float64) for x in (beta, m1, m2))
    g, h = np.asarray(ghat, dtype=np.float64), np.asarray(ghat2, dtype=np.float64)
    m1 = beta1 * m1 + (1.0 - beta1) * g
    m2 = beta2 * m2 + (1.0 - beta2) * h * h
    step = lr * (m1 / (1.0 - beta1 ** t)) / (np.sqrt(m2 / (1.0 - beta2 ** t)) + eps)
    return beta - step, m1, m2
