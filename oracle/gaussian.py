"""Diagonal Gaussian policy head: log-density, entropy, KL (fp64).

PPO for continuous control (Sec. 2.1) uses a Gaussian with state-independent
log standard deviation: sigma = exp(log_std), a = mu + sigma * eps.

Oracle code: test infrastructure only.
"""
import numpy as np

LOG_2PI = np.log(2.0 * np.pi)


def log_prob(a, mu, sigma):
    """log N(a; mu, diag(sigma^2)) summed over the last axis."""
    a, mu, sigma = (np.asarray(v, np.float64) for v in (a, mu, sigma))
    zscore = (a - mu) / sigma
    A = a.shape[-1]
    return -0.5 * np.sum(zscore ** 2, axis=-1) - np.sum(np.log(sigma) * np.ones_like(a), axis=-1) - 0.5 * A * LOG_2PI


def entropy(sigma):
    """Differential entropy sum_j (1/2 + 1/2 log 2 pi + log sigma_j)."""
    sigma = np.asarray(sigma, np.float64)
    return np.sum(0.5 + 0.5 * LOG_2PI + np.log(sigma), axis=-1)


def kl_old_new(mu_old, sigma_old, mu_new, sigma_new):
    """KL( N(mu_old, sigma_old^2) || N(mu_new, sigma_new^2) ) summed over action dims."""
    mu_old, sigma_old, mu_new, sigma_new = (np.asarray(v, np.float64) for v in (mu_old, sigma_old, mu_new, sigma_new))
    return np.sum(np.log(sigma_new / sigma_old)
                  + (sigma_old ** 2 + (mu_old - mu_new) ** 2) / (2.0 * sigma_new ** 2) - 0.5, axis=-1)
