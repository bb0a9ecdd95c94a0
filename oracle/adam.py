"""Global gradient-norm clipping and the Adam step (fp64).

Adam as published (Kingma & Ba 2015), no weight decay, no amsgrad; the bias
corrected step adds eps after the square root:

    t <- t + 1;  m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2
    theta <- theta - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)

Clipping: one L2 norm over every trainable tensor; g <- g * min(1, c / (norm + 1e-6)).

Oracle code: test infrastructure only.
"""
import numpy as np


def global_norm(grads):
    return float(np.sqrt(sum(float(np.sum(np.asarray(g, np.float64) ** 2)) for g in grads)))


def clip_scale(norm, max_norm):
    if max_norm is None or max_norm <= 0 or np.isinf(max_norm):
        return 1.0
    return min(1.0, max_norm / (norm + 1e-6))


def adam_step(theta, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One step; t is the step count *before* this step.  Returns (theta, m, v, t+1)."""
    t = t + 1
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    theta = theta - lr * m_hat / (np.sqrt(v_hat) + eps)
    return theta, m, v, t
