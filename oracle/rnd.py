"""Random network distillation: intrinsic reward with running-variance normalisation (fp64).

Sec. 2.2: curiosity reward = prediction error of a trained predictor against a
frozen random target network, evaluated on a chosen subset of the state.

    x = obs[:, subset];  r_raw_n = sum_k (pred(x_n) - target(x_n))_k^2
    (mean, var, count) <- parallel merge with the N new r_raw values (Chan et al. 1983)
    r_int = r_raw / sqrt(var + 1e-8);   rewards += weight * r_int

Oracle code: test infrastructure only.
"""
import numpy as np

from . import mlp


def raw_error(pred_flat, targ_flat, dims, obs, subset=None, alpha=1.0):
    x = np.asarray(obs, np.float64)
    if subset is not None:
        x = x[:, np.asarray(subset)]
    yp, _ = mlp.forward(mlp.unpack(pred_flat, dims), x, alpha)
    yt, _ = mlp.forward(mlp.unpack(targ_flat, dims), x, alpha)
    return np.sum((yp - yt) ** 2, axis=1)


def merge_running(running, batch):
    """running = (mean, var, count); population variance; Chan et al. pairwise merge."""
    mean, var, count = (float(v) for v in running)
    b = np.asarray(batch, np.float64)
    nb, mb, vb = float(b.size), float(b.mean()), float(b.var())
    tot = count + nb
    delta = mb - mean
    new_mean = mean + delta * nb / tot
    m2 = var * count + vb * nb + delta * delta * count * nb / tot
    return new_mean, m2 / tot, tot


def intrinsic_reward(pred_flat, targ_flat, dims, obs, running, subset=None, update_stats=True, alpha=1.0):
    """Returns (r_int[N], r_raw[N], new running stats)."""
    raw = raw_error(pred_flat, targ_flat, dims, obs, subset, alpha)
    if update_stats:
        running = merge_running(running, raw)
    return raw / np.sqrt(running[1] + 1e-8), raw, running
