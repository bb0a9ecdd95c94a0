"""Pins for oracle.gru and oracle.recurrent: a library GRU (torch, CPU, fp64) for the cell and the reset-free
sequence, closed forms, reset semantics by brute force over separately run episodes, finite differences and
library autodiff for back-propagation through time, finite differences of the whole recurrent PPO loss."""
import numpy as np
import pytest
import torch

from oracle import gru, mlp, recurrent, ppo, rng, bc


def _rand_gru(g, D, H, scale=0.5):
    return scale * g.standard_normal(gru.n_params(D, H))


def _torch_cell(flat, D, H):
    W_ih, b_ih, W_hh, b_hh = gru.unpack(flat, D, H)
    c = torch.nn.GRUCell(D, H).double()
    with torch.no_grad():
        c.weight_ih.copy_(torch.from_numpy(W_ih.T.copy())); c.bias_ih.copy_(torch.from_numpy(b_ih))
        c.weight_hh.copy_(torch.from_numpy(W_hh.T.copy())); c.bias_hh.copy_(torch.from_numpy(b_hh))
    return c


def test_cell_matches_library_gru_cell():
    g = np.random.default_rng(0)
    D, H, n = 5, 7, 9
    flat = _rand_gru(g, D, H)
    x, h = g.standard_normal((n, D)), g.standard_normal((n, H))
    got, _ = gru.cell(gru.unpack(flat, D, H), x, h)
    want = _torch_cell(flat, D, H)(torch.from_numpy(x), torch.from_numpy(h)).detach().numpy()
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_cell_closed_forms():
    D, H, n = 3, 4, 6
    g = np.random.default_rng(1)
    x, h = g.standard_normal((n, D)), g.standard_normal((n, H))
    # all-zero parameters: r = z = 1/2, n = 0  =>  h' = h / 2, and T steps halve T times
    p0 = gru.unpack(np.zeros(gru.n_params(D, H)), D, H)
    np.testing.assert_allclose(gru.cell(p0, x, h)[0], 0.5 * h, rtol=1e-15)
    Hs, _ = gru.sequence_forward(p0, np.zeros((5, n, D)), h, np.zeros((5, n)))
    np.testing.assert_allclose(Hs[4], h / 32.0, rtol=1e-14)
    # update gate saturated open (z = 1): the state is held whatever the input
    W_ih, b_ih, W_hh, b_hh = gru.unpack(_rand_gru(g, D, H), D, H)
    b_hold = b_ih.copy(); b_hold[H:2 * H] = 60.0
    np.testing.assert_allclose(gru.cell((W_ih, b_hold, W_hh, b_hh), x, h)[0], h, rtol=1e-12)
    # update gate shut (z = 0) and reset gate shut (r = 0): h' = tanh(x W_in + b_in), the hidden side drops out
    b_new = b_ih.copy(); b_new[:2 * H] = -60.0
    want = np.tanh(x @ W_ih[:, 2 * H:] + b_new[2 * H:])
    np.testing.assert_allclose(gru.cell((W_ih, b_new, W_hh, b_hh), x, h)[0], want, rtol=1e-12, atol=1e-14)


def test_sequence_without_resets_matches_library_gru():
    g = np.random.default_rng(2)
    D, H, n, T = 4, 6, 5, 7
    flat = _rand_gru(g, D, H)
    W_ih, b_ih, W_hh, b_hh = gru.unpack(flat, D, H)
    net = torch.nn.GRU(D, H).double()
    with torch.no_grad():
        net.weight_ih_l0.copy_(torch.from_numpy(W_ih.T.copy())); net.bias_ih_l0.copy_(torch.from_numpy(b_ih))
        net.weight_hh_l0.copy_(torch.from_numpy(W_hh.T.copy())); net.bias_hh_l0.copy_(torch.from_numpy(b_hh))
    X, h0 = g.standard_normal((T, n, D)), g.standard_normal((n, H))
    Hs, _ = gru.sequence_forward(gru.unpack(flat, D, H), X, h0, np.zeros((T, n)))
    want, _ = net(torch.from_numpy(X), torch.from_numpy(h0)[None])
    np.testing.assert_allclose(Hs, want.detach().numpy(), rtol=1e-11, atol=1e-13)


def _episodes(dones_col):
    """[(start, end)) step ranges of one environment column: a new episode starts after every done."""
    T = len(dones_col)
    out, s = [], 0
    for t in range(T):
        if dones_col[t] and t + 1 < T:
            out.append((s, t + 1)); s = t + 1
    out.append((s, T))
    return out


def test_resets_equal_separately_run_episodes_forward_and_backward():
    """Brute force: cut every environment column at its dones, run each piece on its own (first piece from h0,
    the others from zero) with plain cell steps and plain per-piece back-propagation, and add the gradients up."""
    g = np.random.default_rng(3)
    D, H, n, T = 3, 4, 6, 9
    flat = _rand_gru(g, D, H)
    p = gru.unpack(flat, D, H)
    X, h0 = g.standard_normal((T, n, D)), g.standard_normal((n, H))
    dones = (g.random((T, n)) < 0.3).astype(np.uint8)
    dones[T - 1, 0] = 1                                # a done on the last step has no effect inside the roll-out
    assert dones[:-1].sum() >= 4
    dHs = g.standard_normal((T, n, H))
    Hs, caches = gru.sequence_forward(p, X, h0, dones)
    grad, dh0 = gru.sequence_backward(p, caches, dones, dHs)
    want_H = np.zeros_like(Hs); want_g = np.zeros_like(grad); want_dh0 = np.zeros_like(h0)
    for i in range(n):
        for k, (s, e) in enumerate(_episodes(dones[:, i])):
            h = h0[i:i + 1] if k == 0 else np.zeros((1, H))
            cs = []
            for t in range(s, e):
                h, c = gru.cell(p, X[t, i:i + 1], h)
                want_H[t, i] = h[0]; cs.append(c)
            carry = np.zeros((1, H))
            for t in range(e - 1, s - 1, -1):
                gq, _, carry = gru.cell_backward(p, cs[t - s], dHs[t, i:i + 1] + carry)
                want_g += gru.pack(*gq)
            if k == 0:
                want_dh0[i] = carry[0]
    np.testing.assert_allclose(Hs, want_H, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(grad, want_g, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dh0, want_dh0, rtol=1e-11, atol=1e-14)
    # what happened before a reset cannot be seen after it
    i = int(np.argmax(dones[:-1].sum(axis=0) > 0)); t = int(np.argmax(dones[:-1, i])) + 1
    X2, h02 = X.copy(), h0.copy()
    X2[:t, i] += 1.0; h02[i] -= 2.0
    Hs2, _ = gru.sequence_forward(p, X2, h02, dones)
    assert np.array_equal(Hs2[t:, i], Hs[t:, i]) and not np.allclose(Hs2[:t, i], Hs[:t, i])


def test_bptt_matches_finite_differences_and_library_autodiff():
    g = np.random.default_rng(4)
    D, H, n, T = 3, 5, 4, 6
    flat = _rand_gru(g, D, H)
    X, h0 = g.standard_normal((T, n, D)), g.standard_normal((n, H))
    dones = (g.random((T, n)) < 0.25).astype(np.uint8)
    C = g.standard_normal((T, n, H))

    def scalar(fl, h_init):
        return float(np.sum(C * gru.sequence_forward(gru.unpack(fl, D, H), X, h_init, dones)[0]))

    p = gru.unpack(flat, D, H)
    _, caches = gru.sequence_forward(p, X, h0, dones)
    grad, dh0 = gru.sequence_backward(p, caches, dones, C)
    h = 1e-6
    for k in g.choice(flat.size, size=40, replace=False):
        d = np.zeros_like(flat); d[k] = h
        fd = (scalar(flat + d, h0) - scalar(flat - d, h0)) / (2 * h)
        assert abs(fd - grad[k]) <= 1e-7 * max(1.0, abs(fd)), (k, fd, grad[k])
    for (i, j) in [(0, 0), (1, 3), (3, 4)]:
        d = np.zeros_like(h0); d[i, j] = h
        fd = (scalar(flat, h0 + d) - scalar(flat, h0 - d)) / (2 * h)
        assert abs(fd - dh0[i, j]) <= 1e-7 * max(1.0, abs(fd))
    # library autodiff through library cells with the same resets
    cell = _torch_cell(flat, D, H)
    ht = torch.from_numpy(h0)
    tot = 0.0
    for t in range(T):
        if t > 0:
            ht = ht * torch.from_numpy(1.0 - dones[t - 1].astype(np.float64))[:, None]
        ht = cell(torch.from_numpy(X[t]), ht)
        tot = tot + (torch.from_numpy(C[t]) * ht).sum()
    tot.backward()
    W_ih, b_ih, W_hh, b_hh = gru.unpack(grad, D, H)
    np.testing.assert_allclose(W_ih, cell.weight_ih.grad.numpy().T, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(b_ih, cell.bias_ih.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(W_hh, cell.weight_hh.grad.numpy().T, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(b_hh, cell.bias_hh.grad.numpy(), rtol=1e-10, atol=1e-12)


def _tiny_problem(seed=5, T=5, N=8, D=4, H=6, A=3, hidden=(7,)):
    g = np.random.default_rng(seed)
    dims_a, dims_c = (H,) + hidden + (A,), (H,) + hidden + (1,)
    actor = np.concatenate([_rand_gru(g, D, H), 0.4 * g.standard_normal(mlp.n_params(dims_a)), 0.1 * g.standard_normal(A)])
    critic = np.concatenate([_rand_gru(g, D, H), 0.4 * g.standard_normal(mlp.n_params(dims_c))])
    obs = g.standard_normal((T, N, D))
    dones = (g.random((T, N)) < 0.2).astype(np.uint8)
    h_a, h_c = 0.3 * g.standard_normal((N, H)), 0.3 * g.standard_normal((N, H))
    ro = dict(obs_a=obs, obs_c=obs, dones=dones, h0_a=h_a.copy(), h0_c=h_c.copy())
    acc = {k: [] for k in ("actions", "logp", "values", "mu", "sigma")}
    reset = np.zeros(N)
    for t in range(T):
        o = recurrent.act(actor, critic, D, D, H, dims_a, dims_c, obs[t], obs[t], h_a, h_c, reset, rng.act_noise(1, t, N, A))
        for k in acc:
            acc[k].append(o[k])
        h_a, h_c, reset = o["h_a"], o["h_c"], dones[t]
    ro.update({k: np.stack(v) for k, v in acc.items()})
    ro["adv"] = g.standard_normal((T, N)); ro["returns"] = ro["values"] + 0.3 * g.standard_normal((T, N))
    return dict(actor=actor, critic=critic, D=D, H=H, dims_a=dims_a, dims_c=dims_c, ro=ro, T=T, N=N, A=A)


def test_act_carries_and_resets_the_state_like_the_sequence():
    """Stepping act() with reset = previous dones reproduces the sequence forward from the same h0, so the update
    re-runs exactly what the roll-out computed; on-policy the re-evaluated log-densities equal the stored ones."""
    P = _tiny_problem()
    ro, D, H = P["ro"], P["D"], P["H"]
    ga, ma = recurrent.split(P["actor"], D, H)
    Hs, _ = gru.sequence_forward(gru.unpack(ga, D, H), ro["obs_a"], ro["h0_a"], ro["dones"])
    layers, log_std = mlp.unpack(ma, P["dims_a"], log_std=True)
    mu, _ = mlp.forward(layers, Hs.reshape(-1, H))
    np.testing.assert_allclose(mu.reshape(ro["mu"].shape), ro["mu"], rtol=1e-12, atol=1e-14)
    cfg = ppo.PPOConfig(minibatches=1, epochs=1)
    terms, _, _ = recurrent.minibatch_loss_and_grads(P["actor"], P["critic"], D, D, H, P["dims_a"], P["dims_c"], ro, cfg)
    assert abs(terms["kl"]) < 1e-12 and terms["clip_frac"] == 0.0
    assert abs(terms["surrogate"] + np.mean(ro["adv"])) < 1e-12          # ratio == 1 everywhere


def test_recurrent_loss_gradient_matches_finite_differences():
    P = _tiny_problem(seed=6)
    D, H, ro = P["D"], P["H"], P["ro"]
    g = np.random.default_rng(0)
    # move off the collecting policy so that ratios differ from one and some are clipped
    actor = P["actor"] + 0.05 * g.standard_normal(P["actor"].size)
    critic = P["critic"] + 0.05 * g.standard_normal(P["critic"].size)
    cfg = ppo.PPOConfig(minibatches=1, epochs=1, clip=0.1, value_coef=0.7, entropy_coef=0.02)
    terms, g_a, g_c = recurrent.minibatch_loss_and_grads(actor, critic, D, D, H, P["dims_a"], P["dims_c"], ro, cfg)
    assert 0.0 < terms["clip_frac"] < 1.0

    def loss(a, c):
        return recurrent.minibatch_loss_and_grads(a, c, D, D, H, P["dims_a"], P["dims_c"], ro, cfg)[0]["loss"]

    h = 1e-6
    ng = gru.n_params(D, H)
    picks_a = list(g.choice(ng, 15, replace=False)) + list(ng + g.choice(actor.size - ng, 10, replace=False)) + [actor.size - 1]
    for k in picks_a:
        d = np.zeros_like(actor); d[k] = h
        fd = (loss(actor + d, critic) - loss(actor - d, critic)) / (2 * h)
        assert abs(fd - g_a[k]) <= 2e-6 * max(1e-2, abs(fd)), ("actor", k, fd, g_a[k])
    for k in list(g.choice(ng, 15, replace=False)) + list(ng + g.choice(critic.size - ng, 8, replace=False)):
        d = np.zeros_like(critic); d[k] = h
        fd = (loss(actor, critic + d) - loss(actor, critic - d)) / (2 * h)
        assert abs(fd - g_c[k]) <= 2e-6 * max(1e-2, abs(fd)), ("critic", k, fd, g_c[k])


def test_recurrent_update_minibatches_are_whole_environment_columns():
    P = _tiny_problem(seed=7)
    D, H, ro, N = P["D"], P["H"], P["ro"], P["N"]
    na, nc = P["actor"].size, P["critic"].size
    opt = dict(m_a=np.zeros(na), v_a=np.zeros(na), m_c=np.zeros(nc), v_c=np.zeros(nc), step=0)
    cfg = ppo.PPOConfig(minibatches=4, epochs=2, lr=0.0, seed=9, call_index=2)
    res = recurrent.ppo_update(P["actor"], P["critic"], D, D, H, P["dims_a"], P["dims_c"], ro, cfg, opt, record=True)
    assert res["opt"]["step"] == 8 and res["stats"].shape == (8, 8)
    assert np.array_equal(res["actor"], P["actor"])                     # lr = 0
    for e in range(2):
        assert np.array_equal(np.sort(res["perms"][e]), np.arange(N))
        assert np.array_equal(res["perms"][e], rng.permutation(9, 2, e, N))
    # a minibatch's loss terms are those of its environment columns, in any order of the columns
    envs = res["trace"][5]["envs"]
    assert np.array_equal(envs, res["perms"][1][2:4])
    sub = {k: (v[envs[::-1]] if k in ("h0_a", "h0_c") else v[:, envs[::-1]]) for k, v in ro.items()}
    terms, g_a, _ = recurrent.minibatch_loss_and_grads(P["actor"], P["critic"], D, D, H, P["dims_a"], P["dims_c"], sub,
                                                       ppo.PPOConfig(minibatches=1))
    assert abs(terms["surrogate"] - res["stats"][5, 0]) < 1e-13 and abs(terms["value_loss"] - res["stats"][5, 1]) < 1e-13
    np.testing.assert_allclose(g_a, res["trace"][5]["g_actor"], rtol=1e-10, atol=1e-14)
    # with a learning rate the first step moves every parameter by about lr (Adam's first step is lr * sign(g))
    cfg2 = ppo.PPOConfig(minibatches=4, epochs=1, lr=1e-3, seed=9, call_index=2, max_grad_norm=1e9)
    res2 = recurrent.ppo_update(P["actor"], P["critic"], D, D, H, P["dims_a"], P["dims_c"], ro, cfg2, opt, record=True)
    step1 = res2["trace"][0]["actor"] - P["actor"]
    g1 = res2["trace"][0]["g_actor"]
    big = np.abs(g1) > 1e-6
    np.testing.assert_allclose(step1[big], -1e-3 * np.sign(g1[big]), rtol=1e-3)


def _tiny_distill(seed=8, T=6, N=8, D=4, H=6, A=3, hidden=(7,)):
    g = np.random.default_rng(seed)
    dims = (H,) + hidden + (A,)
    student = np.concatenate([_rand_gru(g, D, H), 0.4 * g.standard_normal(mlp.n_params(dims))])
    obs = g.standard_normal((T, N, D))
    dones = (g.random((T, N)) < 0.25).astype(np.uint8)
    return dict(student=student, D=D, H=H, dims=dims, T=T, N=N, A=A,
                ro=dict(obs=obs, targets=g.standard_normal((T, N, A)), dones=dones, h0=0.3 * g.standard_normal((N, H))))


def test_recurrent_bc_zero_loss_on_own_rollout_and_finite_differences():
    P = _tiny_distill()
    D, H, ro = P["D"], P["H"], P["ro"]
    # targets = what the student itself outputs when stepped through the roll-out with resets: zero loss, zero gradient
    h, reset, outs = ro["h0"], np.zeros(P["N"]), []
    for t in range(P["T"]):
        a, h, hin = recurrent.bc_collect_step(P["student"], D, H, P["dims"], ro["obs"][t], h, reset)
        if t == 0:
            assert np.array_equal(hin, ro["h0"])
        outs.append(a); reset = ro["dones"][t]
    own = dict(ro, targets=np.stack(outs))
    loss, grad = recurrent.bc_minibatch_loss_and_grad(P["student"], D, H, P["dims"], own)
    assert loss < 1e-28 and np.abs(grad).max() < 1e-13
    # finite differences of the scalar loss on random targets
    loss, grad = recurrent.bc_minibatch_loss_and_grad(P["student"], D, H, P["dims"], ro)
    g = np.random.default_rng(0)
    f = lambda s: recurrent.bc_minibatch_loss_and_grad(s, D, H, P["dims"], ro)[0]
    for k in g.choice(P["student"].size, 40, replace=False):
        d = np.zeros_like(P["student"]); d[k] = 1e-6
        fd = (f(P["student"] + d) - f(P["student"] - d)) / 2e-6
        assert abs(fd - grad[k]) <= 1e-6 * max(1e-2, abs(fd)), (k, fd, grad[k])
    # without a memory effect (update gate shut: h' = n, reset gate shut: hidden side dropped) the loss is that of a
    # feed-forward net tanh(x W_in + b_in) -> MLP, which oracle.bc covers
    W_ih, b_ih, W_hh, b_hh = gru.unpack(P["student"][:gru.n_params(D, H)], D, H)
    b_ih = b_ih.copy(); b_ih[:2 * H] = -60.0
    frozen = np.concatenate([gru.pack(W_ih, b_ih, W_hh, b_hh), P["student"][gru.n_params(D, H):]])
    loss_r, _ = recurrent.bc_minibatch_loss_and_grad(frozen, D, H, P["dims"], ro)
    feat = np.tanh(ro["obs"].reshape(-1, D) @ W_ih[:, 2 * H:] + b_ih[2 * H:])
    loss_f, _ = bc.bc_loss_and_grad(P["student"][gru.n_params(D, H):], P["dims"], feat, ro["targets"].reshape(-1, P["A"]))
    assert abs(loss_r - loss_f) < 1e-12


def test_recurrent_bc_update_columns_and_first_step():
    P = _tiny_distill(seed=9)
    n = P["student"].size
    cfg = bc.BCConfig(epochs=2, minibatches=4, lr=1e-3, seed=4, call_index=1)
    res = recurrent.bc_update(P["student"], P["D"], P["H"], P["dims"], P["ro"], cfg, dict(m=np.zeros(n), v=np.zeros(n), step=0), record=True)
    assert res["opt"]["step"] == 8 and res["stats"].shape == (8, 2)
    perm = rng.permutation(4, 1, 1, P["N"])
    assert np.array_equal(res["trace"][6]["envs"], perm[4:6])
    tr = res["trace"][0]
    sub = {k: (v[tr["envs"]] if k == "h0" else v[:, tr["envs"]]) for k, v in P["ro"].items()}
    loss, g = recurrent.bc_minibatch_loss_and_grad(P["student"], P["D"], P["H"], P["dims"], sub)
    assert abs(loss - res["stats"][0, 0]) < 1e-14
    big = np.abs(g) > 1e-4          # Adam's first step is lr * g / (|g| + eps): within 1e-3 of lr * sign(g) there
    np.testing.assert_allclose((tr["student"] - P["student"])[big], -1e-3 * np.sign(g[big]), rtol=1e-3)
