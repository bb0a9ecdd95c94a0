"""Long short-term memory cell: one step, a roll-out-long sequence with episode resets, and back-propagation
through time (fp64).  Same interface as oracle.gru, with the state packed as [h | c] (width 2H).

The paper (Sec. 3) supports recurrent networks without printing a cell; next to the GRU (oracle.gru) this is the
LSTM of Hochreiter & Schmidhuber 1997 with the forget gate of Gers et al. 2000, no peepholes:

    a = x W_ih + b_ih + h W_hh + b_hh                      ([*, 4H], gate order i, f, g, o)
    i = sigmoid(a_i), f = sigmoid(a_f), g = tanh(a_g), o = sigmoid(a_o)
    c' = f * c + i * g;    h' = o * tanh(c')

Sequence with resets: both h and c of an environment are zeroed on the step after its episode ended;
(h0, c0) carried in from the previous roll-out is a constant of the update.

Flat parameter layout (an interface of the library, restated here, not shared code):
W_ih [D, 4H] row-major, b_ih [4H], W_hh [H, 4H] row-major, b_hh [4H].

Oracle code: test infrastructure only.
"""
import numpy as np

GATES = 4


def state_width(H):
    return 2 * H


def n_params(D, H):
    return D * 4 * H + 4 * H + H * 4 * H + 4 * H


def unpack(flat, D, H):
    flat = np.asarray(flat, np.float64)
    assert flat.size == n_params(D, H), (flat.size, n_params(D, H))
    o = 0
    W_ih = flat[o:o + D * 4 * H].reshape(D, 4 * H).copy(); o += D * 4 * H
    b_ih = flat[o:o + 4 * H].copy(); o += 4 * H
    W_hh = flat[o:o + H * 4 * H].reshape(H, 4 * H).copy(); o += H * 4 * H
    b_hh = flat[o:o + 4 * H].copy()
    return W_ih, b_ih, W_hh, b_hh


def pack(W_ih, b_ih, W_hh, b_hh):
    return np.concatenate([np.asarray(a, np.float64).ravel() for a in (W_ih, b_ih, W_hh, b_hh)])


def _sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def cell(p, x, s):
    """One step on the packed state s = [h | c].  Returns (s_new, cache); the new hidden state is s_new[:, :H]."""
    W_ih, b_ih, W_hh, b_hh = p
    H = W_hh.shape[0]
    x = np.asarray(x, np.float64); s = np.asarray(s, np.float64)
    h, c = s[:, :H], s[:, H:]
    a = x @ W_ih + b_ih + h @ W_hh + b_hh
    i, f, g, o = _sigmoid(a[:, :H]), _sigmoid(a[:, H:2 * H]), np.tanh(a[:, 2 * H:3 * H]), _sigmoid(a[:, 3 * H:])
    c_new = f * c + i * g
    tc = np.tanh(c_new)
    h_new = o * tc
    return np.concatenate([h_new, c_new], axis=1), dict(x=x, h=h, c=c, i=i, f=f, g=g, o=o, tc=tc)


def hidden(s, H):
    return np.asarray(s)[..., :H]


def cell_backward(p, cache, ds_new):
    """ds_new = derivative w.r.t. the packed new state [h' | c'].  Returns ((dW_ih, db_ih, dW_hh, db_hh), dx, ds)."""
    W_ih, _, W_hh, _ = p
    x, h, c, i, f, g, o, tc = (cache[k] for k in ("x", "h", "c", "i", "f", "g", "o", "tc"))
    H = h.shape[1]
    dh_new, dc_new = ds_new[:, :H], ds_new[:, H:]
    do = dh_new * tc
    dc_tot = dc_new + dh_new * o * (1.0 - tc * tc)
    da = np.concatenate([dc_tot * g * i * (1.0 - i), dc_tot * c * f * (1.0 - f), dc_tot * i * (1.0 - g * g),
                         do * o * (1.0 - o)], axis=1)
    dh = da @ W_hh.T
    dc = dc_tot * f
    return (x.T @ da, da.sum(axis=0), h.T @ da, da.sum(axis=0)), da @ W_ih.T, np.concatenate([dh, dc], axis=1)


def sequence_forward(p, X, s0, dones):
    """X [T, n, D], s0 [n, 2H], dones [T, n] -> (Hs [T, n, H], caches)."""
    X = np.asarray(X, np.float64)
    H = p[2].shape[0]
    s = np.asarray(s0, np.float64)
    Hs, caches = [], []
    for t in range(X.shape[0]):
        if t > 0:
            s = s * (1.0 - np.asarray(dones[t - 1], np.float64))[:, None]
        s, cch = cell(p, X[t], s)
        Hs.append(s[:, :H]); caches.append(cch)
    return np.stack(Hs), caches


def sequence_backward(p, caches, dones, dHs):
    """dHs [T, n, H]: derivative w.r.t. every h_t through paths outside the recurrence.  Returns (flat gradient,
    ds0 [n, 2H])."""
    T = len(caches)
    H = p[2].shape[0]
    acc = None
    carry = np.zeros((np.asarray(dHs[0]).shape[0], 2 * H))
    for t in range(T - 1, -1, -1):
        ds_new = carry.copy()
        ds_new[:, :H] += np.asarray(dHs[t], np.float64)
        g, _, ds_in = cell_backward(p, caches[t], ds_new)
        acc = g if acc is None else tuple(a + b for a, b in zip(acc, g))
        carry = ds_in * (1.0 - np.asarray(dones[t - 1], np.float64))[:, None] if t > 0 else ds_in
    return pack(*acc), carry
