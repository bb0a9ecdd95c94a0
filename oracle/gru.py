"""Gated recurrent unit: one step, a roll-out-long sequence with episode resets, and backpropagation through
time (fp64).

The paper (Sec. 3) supports recurrent networks with explicit hidden-state management across roll-outs and
back-propagation through time, without printing the cell.  The cell used here is the gated recurrent unit of
Cho et al. 2014 in the form in which the reset gate multiplies the hidden-side candidate term (bias included):

    gi = x W_ih + b_ih,   gh = h W_hh + b_hh              (each [*, 3H], gate order r, z, n)
    r  = sigmoid(gi_r + gh_r);  z = sigmoid(gi_z + gh_z);  n = tanh(gi_n + r * gh_n)
    h' = (1 - z) * n + z * h

Sequence with resets: an episode that ends at step t - 1 (done[t-1] = 1) starts step t from a zero state,

    hin_0 = h0;   hin_t = h_{t-1} * (1 - done[t-1])  (t >= 1);   h_t = cell(x_t, hin_t)

so no gradient crosses an episode boundary, and h0 (the state carried in from the previous roll-out) is a
constant of the update (truncated back-propagation at the roll-out start).

Flat parameter layout (an interface of the library, restated here, not shared code):
W_ih [D, 3H] row-major, b_ih [3H], W_hh [H, 3H] row-major, b_hh [3H].

Oracle code: test infrastructure only.
"""
import numpy as np


GATES = 3


def state_width(H):
    return H


def hidden(s, H):
    return np.asarray(s)[..., :H]


def n_params(D, H):
    return D * 3 * H + 3 * H + H * 3 * H + 3 * H


def unpack(flat, D, H):
    flat = np.asarray(flat, np.float64)
    assert flat.size == n_params(D, H), (flat.size, n_params(D, H))
    o = 0
    W_ih = flat[o:o + D * 3 * H].reshape(D, 3 * H).copy(); o += D * 3 * H
    b_ih = flat[o:o + 3 * H].copy(); o += 3 * H
    W_hh = flat[o:o + H * 3 * H].reshape(H, 3 * H).copy(); o += H * 3 * H
    b_hh = flat[o:o + 3 * H].copy()
    return W_ih, b_ih, W_hh, b_hh


def pack(W_ih, b_ih, W_hh, b_hh):
    return np.concatenate([np.asarray(a, np.float64).ravel() for a in (W_ih, b_ih, W_hh, b_hh)])


def _sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def cell(p, x, h):
    """One step.  Returns (h_new, cache)."""
    W_ih, b_ih, W_hh, b_hh = p
    H = W_hh.shape[0]
    x = np.asarray(x, np.float64); h = np.asarray(h, np.float64)
    gi = x @ W_ih + b_ih
    gh = h @ W_hh + b_hh
    r = _sigmoid(gi[:, :H] + gh[:, :H])
    z = _sigmoid(gi[:, H:2 * H] + gh[:, H:2 * H])
    n = np.tanh(gi[:, 2 * H:] + r * gh[:, 2 * H:])
    h_new = (1.0 - z) * n + z * h
    return h_new, dict(x=x, h=h, r=r, z=z, n=n, gh_n=gh[:, 2 * H:])


def cell_backward(p, cache, dh_new):
    """Returns ((dW_ih, db_ih, dW_hh, db_hh), dx, dh) for a scalar whose derivative w.r.t. h_new is dh_new."""
    W_ih, _, W_hh, _ = p
    x, h, r, z, n, gh_n = (cache[k] for k in ("x", "h", "r", "z", "n", "gh_n"))
    dn = dh_new * (1.0 - z)
    dz = dh_new * (h - n)
    dh = dh_new * z
    dn_pre = dn * (1.0 - n * n)
    dr = dn_pre * gh_n
    dr_pre = dr * r * (1.0 - r)
    dz_pre = dz * z * (1.0 - z)
    dgi = np.concatenate([dr_pre, dz_pre, dn_pre], axis=1)
    dgh = np.concatenate([dr_pre, dz_pre, dn_pre * r], axis=1)
    dh = dh + dgh @ W_hh.T
    dx = dgi @ W_ih.T
    return (x.T @ dgi, dgi.sum(axis=0), h.T @ dgh, dgh.sum(axis=0)), dx, dh


def sequence_forward(p, X, h0, dones):
    """X [T, n, D], h0 [n, H], dones [T, n] -> (Hs [T, n, H], caches)."""
    X = np.asarray(X, np.float64)
    T = X.shape[0]
    h = np.asarray(h0, np.float64)
    Hs, caches = [], []
    for t in range(T):
        if t > 0:
            h = h * (1.0 - np.asarray(dones[t - 1], np.float64))[:, None]
        h, c = cell(p, X[t], h)
        Hs.append(h); caches.append(c)
    return np.stack(Hs), caches


def sequence_backward(p, caches, dones, dHs):
    """Back-propagation through time.  dHs [T, n, H] = derivative of the scalar w.r.t. every h_t through paths
    outside the recurrence.  Returns (flat gradient in the parameter layout, dh0)."""
    T = len(caches)
    acc = None
    carry = np.zeros_like(np.asarray(dHs[0], np.float64))
    for t in range(T - 1, -1, -1):
        g, _, dh_in = cell_backward(p, caches[t], np.asarray(dHs[t], np.float64) + carry)
        acc = g if acc is None else tuple(a + b for a, b in zip(acc, g))
        carry = dh_in * (1.0 - np.asarray(dones[t - 1], np.float64))[:, None] if t > 0 else dh_in
    return pack(*acc), carry
