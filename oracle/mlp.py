"""Multi-layer perceptron with ELU hidden units: forward and backward (fp64).

The paper's networks (Sec. 3, "Network" component) are MLPs; the workloads fix
ELU hidden activations and linear output heads.  Definition used here:

    h_0 = x;   z_l = h_{l-1} W_l + b_l;   h_l = ELU(z_l) for hidden l;   out = z_L
    ELU(z) = z (z > 0),  alpha (e^z - 1) (z <= 0);   ELU'(z) = 1 (z > 0),  ELU(z) + alpha (z <= 0)

Flat parameter layout (an interface of the library, restated here, not shared
code): for each layer l in order, W_l as [dims[l], dims[l+1]] row-major, then
b_l [dims[l+1]]; an actor's buffer ends with log_std[A].

Oracle code: test infrastructure only.
"""
import numpy as np


def n_params(dims, log_std=False):
    n = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))
    return n + (dims[-1] if log_std else 0)


def unpack(flat, dims, log_std=False):
    """Split a flat buffer into [(W_l, b_l)] (+ log_std) as float64 copies."""
    flat = np.asarray(flat, dtype=np.float64)
    assert flat.size == n_params(dims, log_std), (flat.size, n_params(dims, log_std))
    layers, o = [], 0
    for l in range(len(dims) - 1):
        i, j = dims[l], dims[l + 1]
        W = flat[o:o + i * j].reshape(i, j).copy(); o += i * j
        b = flat[o:o + j].copy(); o += j
        layers.append((W, b))
    if log_std:
        return layers, flat[o:o + dims[-1]].copy()
    return layers


def pack(layers, log_std=None):
    parts = []
    for W, b in layers:
        parts += [np.asarray(W, np.float64).ravel(), np.asarray(b, np.float64).ravel()]
    if log_std is not None:
        parts.append(np.asarray(log_std, np.float64).ravel())
    return np.concatenate(parts)


def elu(z, alpha=1.0):
    return np.where(z > 0, z, alpha * np.expm1(np.minimum(z, 0.0)))


def elu_grad(z, alpha=1.0):
    return np.where(z > 0, 1.0, alpha * np.exp(np.minimum(z, 0.0)))


def forward(layers, x, alpha=1.0):
    """Returns (out, cache); cache holds every layer's input and pre-activation."""
    h = np.asarray(x, dtype=np.float64)
    hs, zs = [], []
    L = len(layers)
    for l, (W, b) in enumerate(layers):
        hs.append(h)
        z = h @ W + b
        zs.append(z)
        h = elu(z, alpha) if l < L - 1 else z
    return h, (hs, zs)


def backward(layers, cache, d_out, alpha=1.0):
    """Gradients of a scalar whose derivative w.r.t. the net output is d_out.

    Returns ([(dW_l, db_l)], dx) with dW_l = h_{l-1}^T dz_l, db_l = column sums
    of dz_l, and dh_{l-1} = dz_l W_l^T, dz_l = dh_l * ELU'(z_l) on hidden layers.
    """
    hs, zs = cache
    L = len(layers)
    grads = [None] * L
    dz = np.asarray(d_out, dtype=np.float64)
    for l in range(L - 1, -1, -1):
        W, _ = layers[l]
        grads[l] = (hs[l].T @ dz, dz.sum(axis=0))
        dh = dz @ W.T
        if l > 0:
            dz = dh * elu_grad(zs[l - 1], alpha)
    return grads, dh
