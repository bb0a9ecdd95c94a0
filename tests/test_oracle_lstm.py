"""Pins for oracle.lstm and the cell="lstm" path of oracle.recurrent: a library LSTM (torch, CPU, fp64) for the
cell and the reset-free sequence, closed forms, resets by brute force over separately run episodes, finite
differences and library autodiff for back-propagation through time, finite differences of the recurrent losses."""
import numpy as np
import torch

from oracle import lstm, mlp, recurrent, ppo, rng, bc


def _rand(g, D, H, scale=0.5):
    return scale * g.standard_normal(lstm.n_params(D, H))


def _torch_cell(flat, D, H):
    W_ih, b_ih, W_hh, b_hh = lstm.unpack(flat, D, H)
    c = torch.nn.LSTMCell(D, H).double()
    with torch.no_grad():
        c.weight_ih.copy_(torch.from_numpy(W_ih.T.copy())); c.bias_ih.copy_(torch.from_numpy(b_ih))
        c.weight_hh.copy_(torch.from_numpy(W_hh.T.copy())); c.bias_hh.copy_(torch.from_numpy(b_hh))
    return c


def test_cell_matches_library_lstm_cell_and_closed_forms():
    g = np.random.default_rng(0)
    D, H, n = 5, 7, 9
    flat = _rand(g, D, H)
    x, s = g.standard_normal((n, D)), g.standard_normal((n, 2 * H))
    got, _ = lstm.cell(lstm.unpack(flat, D, H), x, s)
    h, c = _torch_cell(flat, D, H)(torch.from_numpy(x), (torch.from_numpy(s[:, :H].copy()), torch.from_numpy(s[:, H:].copy())))
    np.testing.assert_allclose(got[:, :H], h.detach().numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(got[:, H:], c.detach().numpy(), rtol=1e-12, atol=1e-13)
    # all-zero parameters: i = f = o = 1/2, g = 0  =>  c' = c / 2, h' = tanh(c / 2) / 2
    p0 = lstm.unpack(np.zeros(lstm.n_params(D, H)), D, H)
    s1, _ = lstm.cell(p0, x, s)
    np.testing.assert_allclose(s1[:, H:], 0.5 * s[:, H:], rtol=1e-15)
    np.testing.assert_allclose(s1[:, :H], 0.5 * np.tanh(0.5 * s[:, H:]), rtol=1e-15)
    # forget gate open, input gate shut: the cell content is held whatever the input
    W_ih, b_ih, W_hh, b_hh = lstm.unpack(flat, D, H)
    b = b_ih.copy(); b[:H] = -60.0; b[H:2 * H] = 60.0
    s2, _ = lstm.cell((W_ih, b, W_hh, b_hh), x, s)
    np.testing.assert_allclose(s2[:, H:], s[:, H:], rtol=1e-12)


def test_sequence_without_resets_matches_library_lstm():
    g = np.random.default_rng(2)
    D, H, n, T = 4, 6, 5, 7
    flat = _rand(g, D, H)
    W_ih, b_ih, W_hh, b_hh = lstm.unpack(flat, D, H)
    net = torch.nn.LSTM(D, H).double()
    with torch.no_grad():
        net.weight_ih_l0.copy_(torch.from_numpy(W_ih.T.copy())); net.bias_ih_l0.copy_(torch.from_numpy(b_ih))
        net.weight_hh_l0.copy_(torch.from_numpy(W_hh.T.copy())); net.bias_hh_l0.copy_(torch.from_numpy(b_hh))
    X, s0 = g.standard_normal((T, n, D)), g.standard_normal((n, 2 * H))
    Hs, _ = lstm.sequence_forward(lstm.unpack(flat, D, H), X, s0, np.zeros((T, n)))
    want, _ = net(torch.from_numpy(X), (torch.from_numpy(s0[:, :H].copy())[None], torch.from_numpy(s0[:, H:].copy())[None]))
    np.testing.assert_allclose(Hs, want.detach().numpy(), rtol=1e-11, atol=1e-13)


def _episodes(dones_col):
    T = len(dones_col)
    out, s = [], 0
    for t in range(T):
        if dones_col[t] and t + 1 < T:
            out.append((s, t + 1)); s = t + 1
    out.append((s, T))
    return out


def test_resets_equal_separately_run_episodes_forward_and_backward():
    g = np.random.default_rng(3)
    D, H, n, T = 3, 4, 6, 9
    flat = _rand(g, D, H)
    p = lstm.unpack(flat, D, H)
    X, s0 = g.standard_normal((T, n, D)), g.standard_normal((n, 2 * H))
    dones = (g.random((T, n)) < 0.3).astype(np.uint8)
    dHs = g.standard_normal((T, n, H))
    Hs, caches = lstm.sequence_forward(p, X, s0, dones)
    grad, ds0 = lstm.sequence_backward(p, caches, dones, dHs)
    want_H = np.zeros_like(Hs); want_g = np.zeros_like(grad); want_ds0 = np.zeros_like(s0)
    for i in range(n):
        for k, (a, e) in enumerate(_episodes(dones[:, i])):
            s = s0[i:i + 1] if k == 0 else np.zeros((1, 2 * H))
            cs = []
            for t in range(a, e):
                s, c = lstm.cell(p, X[t, i:i + 1], s)
                want_H[t, i] = s[0, :H]; cs.append(c)
            carry = np.zeros((1, 2 * H))
            for t in range(e - 1, a - 1, -1):
                d = carry.copy(); d[:, :H] += dHs[t, i:i + 1]
                gq, _, carry = lstm.cell_backward(p, cs[t - a], d)
                want_g += lstm.pack(*gq)
            if k == 0:
                want_ds0[i] = carry[0]
    np.testing.assert_allclose(Hs, want_H, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(grad, want_g, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(ds0, want_ds0, rtol=1e-11, atol=1e-14)


def test_bptt_matches_finite_differences_and_library_autodiff():
    g = np.random.default_rng(4)
    D, H, n, T = 3, 5, 4, 6
    flat = _rand(g, D, H)
    X, s0 = g.standard_normal((T, n, D)), g.standard_normal((n, 2 * H))
    dones = (g.random((T, n)) < 0.25).astype(np.uint8)
    Cw = g.standard_normal((T, n, H))

    def scalar(fl, s_init):
        return float(np.sum(Cw * lstm.sequence_forward(lstm.unpack(fl, D, H), X, s_init, dones)[0]))

    p = lstm.unpack(flat, D, H)
    _, caches = lstm.sequence_forward(p, X, s0, dones)
    grad, ds0 = lstm.sequence_backward(p, caches, dones, Cw)
    h = 1e-6
    for k in g.choice(flat.size, size=40, replace=False):
        d = np.zeros_like(flat); d[k] = h
        fd = (scalar(flat + d, s0) - scalar(flat - d, s0)) / (2 * h)
        assert abs(fd - grad[k]) <= 1e-7 * max(1.0, abs(fd)), (k, fd, grad[k])
    for (i, j) in [(0, 0), (1, 3), (3, 7), (2, 9)]:          # h0 and c0 entries
        d = np.zeros_like(s0); d[i, j] = h
        fd = (scalar(flat, s0 + d) - scalar(flat, s0 - d)) / (2 * h)
        assert abs(fd - ds0[i, j]) <= 1e-7 * max(1.0, abs(fd))
    cell = _torch_cell(flat, D, H)
    ht, ct = torch.from_numpy(s0[:, :H].copy()), torch.from_numpy(s0[:, H:].copy())
    tot = 0.0
    for t in range(T):
        if t > 0:
            keep = torch.from_numpy(1.0 - dones[t - 1].astype(np.float64))[:, None]
            ht, ct = ht * keep, ct * keep
        ht, ct = cell(torch.from_numpy(X[t]), (ht, ct))
        tot = tot + (torch.from_numpy(Cw[t]) * ht).sum()
    tot.backward()
    W_ih, b_ih, W_hh, b_hh = lstm.unpack(grad, D, H)
    np.testing.assert_allclose(W_ih, cell.weight_ih.grad.numpy().T, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(b_ih, cell.bias_ih.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(W_hh, cell.weight_hh.grad.numpy().T, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(b_hh, cell.bias_hh.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_recurrent_ppo_and_bc_losses_with_lstm_memory():
    """The cell="lstm" path of oracle.recurrent: act() stepping reproduces the sequence, on-policy identities hold,
    and the gradients of both losses match finite differences."""
    g = np.random.default_rng(6)
    T, N, D, H, A, hidden = 5, 8, 4, 6, 3, (7,)
    dims_a, dims_c = (H,) + hidden + (A,), (H,) + hidden + (1,)
    actor = np.concatenate([_rand(g, D, H), 0.4 * g.standard_normal(mlp.n_params(dims_a)), 0.1 * g.standard_normal(A)])
    critic = np.concatenate([_rand(g, D, H), 0.4 * g.standard_normal(mlp.n_params(dims_c))])
    obs = g.standard_normal((T, N, D))
    dones = (g.random((T, N)) < 0.2).astype(np.uint8)
    s_a, s_c = 0.3 * g.standard_normal((N, 2 * H)), 0.3 * g.standard_normal((N, 2 * H))
    ro = dict(obs_a=obs, obs_c=obs, dones=dones, h0_a=s_a.copy(), h0_c=s_c.copy())
    acc = {k: [] for k in ("actions", "logp", "values", "mu", "sigma")}
    reset = np.zeros(N)
    for t in range(T):
        o = recurrent.act(actor, critic, D, D, H, dims_a, dims_c, obs[t], obs[t], s_a, s_c, reset, rng.act_noise(1, t, N, A), cell="lstm")
        assert o["h_a"].shape == (N, 2 * H)
        for k in acc:
            acc[k].append(o[k])
        s_a, s_c, reset = o["h_a"], o["h_c"], dones[t]
    ro.update({k: np.stack(v) for k, v in acc.items()})
    ro["adv"] = g.standard_normal((T, N)); ro["returns"] = ro["values"] + 0.3 * g.standard_normal((T, N))
    cfg = ppo.PPOConfig(minibatches=1, epochs=1, clip=0.1, value_coef=0.7, entropy_coef=0.02)
    terms, _, _ = recurrent.minibatch_loss_and_grads(actor, critic, D, D, H, dims_a, dims_c, ro, cfg, cell="lstm")
    assert abs(terms["kl"]) < 1e-12 and abs(terms["surrogate"] + np.mean(ro["adv"])) < 1e-12
    a2 = actor + 0.05 * g.standard_normal(actor.size); c2 = critic + 0.05 * g.standard_normal(critic.size)
    terms, g_a, g_c = recurrent.minibatch_loss_and_grads(a2, c2, D, D, H, dims_a, dims_c, ro, cfg, cell="lstm")
    loss = lambda a, c: recurrent.minibatch_loss_and_grads(a, c, D, D, H, dims_a, dims_c, ro, cfg, cell="lstm")[0]["loss"]
    h = 1e-6
    for k in list(g.choice(a2.size, 25, replace=False)) + [a2.size - 1]:
        d = np.zeros_like(a2); d[k] = h
        fd = (loss(a2 + d, c2) - loss(a2 - d, c2)) / (2 * h)
        assert abs(fd - g_a[k]) <= 2e-6 * max(1e-2, abs(fd)), ("actor", k, fd, g_a[k])
    for k in g.choice(c2.size, 20, replace=False):
        d = np.zeros_like(c2); d[k] = h
        fd = (loss(a2, c2 + d) - loss(a2, c2 - d)) / (2 * h)
        assert abs(fd - g_c[k]) <= 2e-6 * max(1e-2, abs(fd)), ("critic", k, fd, g_c[k])
    # behaviour cloning of an LSTM student
    dims_s = (H,) + hidden + (A,)
    student = np.concatenate([_rand(g, D, H), 0.4 * g.standard_normal(mlp.n_params(dims_s))])
    bro = dict(obs=obs, targets=g.standard_normal((T, N, A)), dones=dones, h0=0.3 * g.standard_normal((N, 2 * H)))
    l0, gs = recurrent.bc_minibatch_loss_and_grad(student, D, H, dims_s, bro, cell="lstm")
    f = lambda s: recurrent.bc_minibatch_loss_and_grad(s, D, H, dims_s, bro, cell="lstm")[0]
    for k in g.choice(student.size, 30, replace=False):
        d = np.zeros_like(student); d[k] = h
        fd = (f(student + d) - f(student - d)) / (2 * h)
        assert abs(fd - gs[k]) <= 1e-6 * max(1e-2, abs(fd)), (k, fd, gs[k])
    n = student.size
    res = recurrent.bc_update(student, D, H, dims_s, bro, bc.BCConfig(epochs=1, minibatches=2, seed=3), dict(m=np.zeros(n), v=np.zeros(n), step=0), cell="lstm")
    assert res["opt"]["step"] == 2 and abs(res["stats"][0, 0] - recurrent.bc_minibatch_loss_and_grad(
        student, D, H, dims_s, {k: (v[rng.permutation(3, 0, 0, N)[:4]] if k == "h0" else v[:, rng.permutation(3, 0, 0, N)[:4]]) for k, v in bro.items()}, cell="lstm")[0]) < 1e-14
