"""Pins for oracle.mlp, oracle.gaussian and oracle.adam."""
from fractions import Fraction
import math
import numpy as np
import scipy.stats as st
from oracle import mlp, gaussian, adam


def _net(dims, seed=0, log_std=False):
    g = np.random.default_rng(seed)
    flat = g.normal(scale=0.5, size=mlp.n_params(dims, log_std))
    return flat


def test_flat_layout_and_single_layer_is_affine():
    dims = (3, 2)
    flat = np.array([1., 2., 3., 4., 5., 6., 10., 20.])   # W = [[1,2],[3,4],[5,6]], b = [10,20]
    (W, b), = mlp.unpack(flat, dims)
    assert W.tolist() == [[1, 2], [3, 4], [5, 6]] and b.tolist() == [10, 20]
    out, _ = mlp.forward([(W, b)], np.array([[1., 0., -1.]]))
    assert out.tolist() == [[1 - 5 + 10, 2 - 6 + 20]]
    assert np.array_equal(mlp.pack([(W, b)]), flat)


def test_elu_values_and_derivative_continuity():
    z = np.array([-1e3, -1.0, -1e-9, 0.0, 1e-9, 2.0])
    y = mlp.elu(z)
    assert y[0] == -1.0 and abs(y[1] - (math.exp(-1) - 1)) < 1e-15 and y[3] == 0.0 and y[5] == 2.0
    d = mlp.elu_grad(z)
    assert d[0] == 0.0 and abs(d[2] - 1.0) < 1e-8 and d[3] == 1.0 and d[4] == 1.0
    np.testing.assert_allclose(d[z <= 0], y[z <= 0] + 1.0, atol=1e-15)      # ELU' = ELU + alpha on z <= 0


def test_two_layer_forward_by_hand():
    # x=[1,-2]; W1=[[1,0],[0,1]], b1=[0,0] -> z=[1,-2] -> h=[1, e^-2 - 1]; W2=[[2],[3]], b2=[1]
    flat = np.array([1., 0., 0., 1., 0., 0., 2., 3., 1.])
    out, _ = mlp.forward(mlp.unpack(flat, (2, 2, 1)), np.array([[1., -2.]]))
    assert abs(out[0, 0] - (2 * 1 + 3 * (math.exp(-2) - 1) + 1)) < 1e-15


def test_backward_matches_central_differences():
    dims = (5, 7, 6, 3)
    flat = _net(dims, 1)
    g = np.random.default_rng(2)
    x = g.normal(size=(4, 5)); c = g.normal(size=(4, 3))

    def f(p):
        out, _ = mlp.forward(mlp.unpack(p, dims), x)
        return float(np.sum(c * out))

    layers = mlp.unpack(flat, dims)
    _, cache = mlp.forward(layers, x)
    grads, dx = mlp.backward(layers, cache, c)
    ana = mlp.pack(grads)
    h = 1e-6
    num = np.array([(f(flat + h * e) - f(flat - h * e)) / (2 * h) for e in np.eye(flat.size)])
    np.testing.assert_allclose(ana, num, rtol=1e-6, atol=1e-8)

    def fx(xx):
        out, _ = mlp.forward(layers, xx.reshape(4, 5))
        return float(np.sum(c * out))
    numx = np.array([(fx(x.ravel() + h * e) - fx(x.ravel() - h * e)) / (2 * h) for e in np.eye(20)])
    np.testing.assert_allclose(dx.ravel(), numx, rtol=1e-6, atol=1e-8)


def test_gaussian_logprob_entropy_kl():
    g = np.random.default_rng(0)
    A = 5
    mu = g.normal(size=(6, A)); sigma = np.exp(g.normal(scale=0.3, size=A)); a = g.normal(size=(6, A))
    want = st.norm.logpdf(a, loc=mu, scale=sigma).sum(axis=1)
    np.testing.assert_allclose(gaussian.log_prob(a, mu, np.broadcast_to(sigma, mu.shape)), want, rtol=1e-13)
    assert abs(gaussian.log_prob(mu[:1], mu[:1], np.ones((1, A)))[0] + 0.5 * A * math.log(2 * math.pi)) < 1e-14
    H = gaussian.entropy(sigma)
    assert abs(H - 0.5 * math.log((2 * math.pi * math.e) ** A * np.prod(sigma ** 2))) < 1e-13
    assert abs(H - st.multivariate_normal(np.zeros(A), np.diag(sigma ** 2)).entropy()) < 1e-12
    # KL against numerical integration in one dimension, and KL(p || p) = 0
    from scipy.integrate import quad
    m0, s0, m1, s1 = 0.3, 0.8, -0.2, 1.3
    num, _ = quad(lambda x: st.norm.pdf(x, m0, s0) * (st.norm.logpdf(x, m0, s0) - st.norm.logpdf(x, m1, s1)), -12, 12)
    assert abs(gaussian.kl_old_new([[m0]], [[s0]], [[m1]], [[s1]])[0] - num) < 1e-9
    assert gaussian.kl_old_new(mu, np.broadcast_to(sigma, mu.shape), mu, np.broadcast_to(sigma, mu.shape)).max() < 1e-15


def test_clip_scale():
    g = [np.array([3.0, 0.0]), np.array([[4.0]])]
    assert abs(adam.global_norm(g) - 5.0) < 1e-15
    s = adam.clip_scale(5.0, 1.0)
    assert abs(s * 5.0 - 1.0) < 1e-6 and adam.clip_scale(0.5, 1.0) == 1.0
    assert adam.clip_scale(5.0, float("inf")) == 1.0 and adam.clip_scale(5.0, 0.0) == 1.0


def test_adam_first_step_and_constant_gradient():
    lr, eps = 0.01, 1e-8
    th, m, v, t = np.array([1.0, -2.0]), np.zeros(2), np.zeros(2), 0
    g = np.array([0.3, -7.0])
    th1, m1, v1, t1 = adam.adam_step(th, g, m, v, t, lr, eps=eps)
    np.testing.assert_allclose(th1, th - lr * g / (np.abs(g) + eps), rtol=1e-13)       # m_hat = g, v_hat = g^2
    assert t1 == 1 and np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.001 * g * g)
    cur = (th, m, v, t)
    for k in range(1, 6):                                                              # constant g: equal steps
        cur = adam.adam_step(cur[0], g, cur[1], cur[2], cur[3], lr, eps=eps)
        np.testing.assert_allclose(cur[0], th - k * lr * g / (np.abs(g) + eps), rtol=1e-12)
    th0, m0, v0, t0 = adam.adam_step(th, g, m, v, t, 0.0)                              # lr = 0
    assert np.array_equal(th0, th) and t0 == 1 and np.all(m0 != 0) and np.all(v0 != 0)


def test_adam_three_hand_steps_exact_rationals():
    """g = 1, -2, 1/2 with lr = 1/10, eps = 0, stepped in exact rational arithmetic."""
    lr, b1, b2 = Fraction(1, 10), Fraction(9, 10), Fraction(999, 1000)
    gs = [Fraction(1), Fraction(-2), Fraction(1, 2)]
    m = v = Fraction(0); theta = 0.0
    th, mm, vv, t = np.array([0.0]), np.zeros(1), np.zeros(1), 0
    for k, g in enumerate(gs, 1):
        m = b1 * m + (1 - b1) * g
        v = b2 * v + (1 - b2) * g * g
        theta -= float(lr * (m / (1 - b1 ** k))) / math.sqrt(float(v / (1 - b2 ** k)))
        th, mm, vv, t = adam.adam_step(th, np.array([float(g)]), mm, vv, t, 0.1, eps=0.0)
        assert abs(th[0] - theta) < 1e-14 and abs(mm[0] - float(m)) < 1e-16 and abs(vv[0] - float(v)) < 1e-16
    assert m == Fraction(-49, 1000) and v == Fraction(999, 1000) * Fraction(4999, 1000000) + Fraction(1, 4000)
    # row 2 of the table by hand: theta_2 = -1/10 + (1/10) (11/19) / sqrt(4999/1999)
    th2 = adam.adam_step(*adam.adam_step(np.array([0.0]), np.array([1.0]), np.zeros(1), np.zeros(1), 0, 0.1, eps=0.0)[:1],
                         np.array([-2.0]), np.array([0.1]), np.array([0.001]), 1, 0.1, eps=0.0)[0]
    assert abs(th2[0] - (-0.1 + 0.1 * (11 / 19) / math.sqrt(4999 / 1999))) < 1e-15
