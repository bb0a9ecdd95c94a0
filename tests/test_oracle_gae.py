"""Pins for oracle.gae: closed forms of GAE(lambda), an O(T^2) double-sum definition, done/timeouts semantics."""
import numpy as np
from oracle import gae as G


def _rand(T=7, N=5, seed=0, p_done=0.0):
    g = np.random.default_rng(seed)
    return (g.normal(size=(T, N)), g.normal(size=(T, N)), g.normal(size=N),
            (g.random((T, N)) < p_done).astype(np.uint8))


def test_lambda_one_is_discounted_return_minus_value():
    r, V, Vl, d = _rand()
    T, N = r.shape
    gamma = 0.9
    adv, ret = G.gae(r, V, Vl, d, gamma, 1.0)
    for t in range(T):
        want = sum(gamma ** k * r[t + k] for k in range(T - t)) + gamma ** (T - t) * Vl
        np.testing.assert_allclose(ret[t], want, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(adv[t], want - V[t], rtol=1e-12, atol=1e-12)


def test_gamma_zero_and_lambda_zero():
    r, V, Vl, d = _rand(p_done=0.3)
    adv, ret = G.gae(r, V, Vl, d, 0.0, 0.7)
    np.testing.assert_allclose(adv, r - V, atol=1e-14)
    np.testing.assert_allclose(ret, r, atol=1e-14)
    adv, _ = G.gae(r, V, Vl, d, 0.95, 0.0)
    Vn = np.vstack([V[1:], Vl[None]])
    np.testing.assert_allclose(adv, r + 0.95 * (1 - d) * Vn - V, atol=1e-14)


def test_bruteforce_double_sum():
    """A_t = sum_{k>=0} (gamma lam)^k delta_{t+k}, truncated at the first done at or after t."""
    r, V, Vl, d = _rand(T=9, N=6, seed=3, p_done=0.25)
    gamma, lam = 0.97, 0.9
    T, N = r.shape
    Vn = np.vstack([V[1:], Vl[None]])
    adv, ret = G.gae(r, V, Vl, d, gamma, lam)
    for n in range(N):
        for t in range(T):
            a = 0.0
            for k in range(T - t):
                s = t + k
                delta = r[s, n] + gamma * (0.0 if d[s, n] else Vn[s, n]) - V[s, n]
                a += (gamma * lam) ** k * delta
                if d[s, n]:
                    break
            assert abs(adv[t, n] - a) < 1e-12
            assert abs(ret[t, n] - (a + V[t, n])) < 1e-12


def test_done_cuts_dependence_on_the_future():
    r, V, Vl, d = _rand(T=8, N=4, seed=5)
    d[:] = 0
    d[3, :] = 1
    a0, r0 = G.gae(r, V, Vl, d, 0.99, 0.95)
    r2, V2 = r.copy(), V.copy()
    r2[4:] += 100.0; V2[4:] -= 50.0
    a1, r1 = G.gae(r2, V2, Vl + 7.0, d, 0.99, 0.95)
    assert np.array_equal(a0[:4], a1[:4]) and np.array_equal(r0[:4], r1[:4])
    assert not np.allclose(a0[4:], a1[4:])


def test_all_dones_and_T1():
    r, V, Vl, d = _rand(T=5, N=3, seed=7)
    adv, ret = G.gae(r, V, Vl, np.ones_like(d), 0.99, 0.95)
    np.testing.assert_allclose(adv, r - V, atol=1e-14)
    adv, ret = G.gae(r[:1], V[:1], Vl, d[:1] * 0, 0.9, 0.5)
    np.testing.assert_allclose(adv[0], r[0] + 0.9 * Vl - V[0], atol=1e-14)


def test_timeout_equals_reward_bootstrap():
    r, V, Vl, d = _rand(T=6, N=5, seed=9, p_done=0.3)
    to = d * (np.random.default_rng(1).random(d.shape) < 0.5)
    a0, r0 = G.gae(r, V, Vl, d, 0.98, 0.9, timeouts=to)
    a1, r1 = G.gae(r + 0.98 * V * to, V, Vl, d, 0.98, 0.9)
    np.testing.assert_allclose(a0, a1, atol=1e-14); np.testing.assert_allclose(r0, r1, atol=1e-14)
    assert not np.allclose(a0, G.gae(r, V, Vl, d, 0.98, 0.9)[0])


def test_normalisation_moments():
    a = np.random.default_rng(2).normal(3.0, 5.0, size=(24, 64))
    z = G.normalize_advantages(a)
    assert abs(z.mean()) < 1e-12 and abs(z.std(ddof=1) - 1.0) < 1e-7
    assert np.all(np.sign(z - z.mean()) == np.sign(a - a.mean()))
