"""Generalised advantage estimation over a [T, N] rollout (fp64).

PPO's return computation (Sec. 2.1; time-limit handling named in Sec. 3).
With V_T := last_values and A_T := 0, for t = T-1 .. 0:

    nd_t    = 1 - done_t
    delta_t = r_t + gamma * nd_t * V_{t+1} - V_t
    A_t     = delta_t + gamma * lam * nd_t * A_{t+1}
    R_t     = A_t + V_t

done_t = 1 means the episode ended with the action taken at t (same-step reset:
the next observation already belongs to a new episode), so it cuts both the
bootstrap and the accumulated advantage.  A time-limit truncation at t first
adds the bootstrap it would otherwise lose:  r_t <- r_t + gamma * V_t * timeout_t.

Oracle code: test infrastructure only.
"""
import numpy as np


def gae(rewards, values, last_values, dones, gamma, lam, timeouts=None):
    r = np.asarray(rewards, np.float64).copy()
    V = np.asarray(values, np.float64)
    d = np.asarray(dones, np.float64)
    T, N = r.shape
    if timeouts is not None:
        r = r + gamma * V * np.asarray(timeouts, np.float64)
    adv = np.zeros((T, N))
    ret = np.zeros((T, N))
    A_next = np.zeros(N)
    V_next = np.asarray(last_values, np.float64)
    for t in range(T - 1, -1, -1):
        nd = 1.0 - d[t]
        delta = r[t] + gamma * nd * V_next - V[t]
        A_next = delta + gamma * lam * nd * A_next
        adv[t] = A_next
        ret[t] = A_next + V[t]
        V_next = V[t]
    return adv, ret


def normalize_advantages(adv, eps=1e-8):
    """(A - mean) / (std + eps) over the whole batch, std with the n-1 divisor."""
    a = np.asarray(adv, np.float64)
    return (a - a.mean()) / (a.std(ddof=1) + eps)
