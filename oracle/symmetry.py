"""Symmetry augmentation and the mirror loss (fp64).

Sec. 2.2: collected data are augmented with mirrored states using the robot's
physical symmetries, and an extra loss can reinforce symmetric behaviour.
A mirror map is a signed permutation:  mirror(x)[j] = sign[j] * x[perm[j]].

Oracle code: test infrastructure only.
"""
import numpy as np


def mirror(x, perm, sign):
    x = np.asarray(x, np.float64)
    return x[..., np.asarray(perm)] * np.asarray(sign, np.float64)


def is_involution(perm, sign):
    perm = np.asarray(perm); sign = np.asarray(sign, np.float64)
    n = perm.size
    if sorted(perm.tolist()) != list(range(n)) or not np.all(np.abs(sign) == 1.0):
        return False
    # mirror(mirror(x))[j] = sign[j] * sign[perm[j]] * x[perm[perm[j]]]
    return bool(np.all(perm[perm] == np.arange(n)) and np.all(sign * sign[perm] == 1.0))


def augment(obs, actions, perm_obs, sign_obs, perm_act, sign_act):
    """out[0:B] = in, out[B:2B] = mirror(in), for observations and actions."""
    obs = np.asarray(obs, np.float64); actions = np.asarray(actions, np.float64)
    return (np.concatenate([obs, mirror(obs, perm_obs, sign_obs)], axis=0),
            np.concatenate([actions, mirror(actions, perm_act, sign_act)], axis=0))


def mirror_loss(mu_orig, mu_on_mirrored_obs, perm_act, sign_act):
    """mean over rows and action dims of (mu(mirror(o)) - mirror_a(mu(o)))^2.

    Returns (loss, d loss / d mu_on_mirrored_obs); the mirrored-mean target is
    treated as a constant (no gradient flows into mu_orig).
    """
    target = mirror(mu_orig, perm_act, sign_act)
    diff = np.asarray(mu_on_mirrored_obs, np.float64) - target
    return float(np.mean(diff ** 2)), 2.0 * diff / diff.size
