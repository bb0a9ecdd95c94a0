"""Pins for oracle.ppo / symmetry / bc / rnd: special cases, finite differences of the scalar loss, invariants."""
import numpy as np
from oracle import mlp, ppo, gaussian, symmetry, bc, rnd, rng, adam

DA, DC, A = 6, 5, 3
DIMS_A, DIMS_C = (DA, 8, 7, A), (DC, 9, 1)


def _setup(seed=0, n=16, perturb=0.0):
    g = np.random.default_rng(seed)
    actor = g.normal(scale=0.4, size=mlp.n_params(DIMS_A, True)); actor[-A:] = g.normal(scale=0.2, size=A)
    critic = g.normal(scale=0.4, size=mlp.n_params(DIMS_C))
    obs_a, obs_c = g.normal(size=(n, DA)), g.normal(size=(n, DC))
    out = ppo.act(actor, critic, DIMS_A, DIMS_C, obs_a, obs_c, g.normal(size=(n, A)))
    batch = dict(obs_a=obs_a, obs_c=obs_c, actions=out["actions"], logp=out["logp"], values=out["values"],
                 mu=out["mu"], sigma=out["sigma"], adv=g.normal(size=n), returns=out["values"] + g.normal(scale=0.3, size=n))
    if perturb:
        actor = actor + perturb * g.normal(size=actor.size); critic = critic + perturb * g.normal(size=critic.size)
    return actor, critic, batch


def _sym(seed=0):
    from workloads import random_involution
    g = np.random.default_rng(seed)
    po, so = random_involution(g, DA); pc, sc = random_involution(g, DC); pa, sa = random_involution(g, A)
    return ppo.SymSpec(po, so, pc, sc, pa, sa, mirror_loss_coef=0.7)


def test_act_outputs():
    actor, critic, b = _setup()
    np.testing.assert_allclose(b["actions"], b["mu"] + b["sigma"] * ((b["actions"] - b["mu"]) / b["sigma"]))
    np.testing.assert_allclose(b["sigma"], np.broadcast_to(np.exp(actor[-A:]), b["mu"].shape))
    z = (b["actions"] - b["mu"]) / b["sigma"]
    np.testing.assert_allclose(b["logp"], -0.5 * (z ** 2).sum(1) - np.log(b["sigma"]).sum(1) - 0.5 * A * np.log(2 * np.pi))


def test_ratio_one_surrogate_is_minus_mean_advantage():
    actor, critic, b = _setup()
    cfg = ppo.PPOConfig()
    terms, ga, gc = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg)
    assert abs(terms["surrogate"] + b["adv"].mean()) < 1e-12
    assert terms["clip_frac"] == 0.0 and abs(terms["kl"]) < 1e-14
    assert abs(terms["value_loss"] - np.mean((b["values"] - b["returns"]) ** 2)) < 1e-12     # V = V_old: branches equal
    assert abs(terms["entropy"] - gaussian.entropy(np.exp(actor[-A:]))) < 1e-14


def test_clipped_sample_has_zero_policy_gradient():
    actor, critic, b = _setup(n=1)
    cfg = ppo.PPOConfig(entropy_coef=0.0, value_coef=0.0)
    b["adv"] = np.array([2.0]); b["logp"] = b["logp"] - 1.0          # ratio = e > 1 + clip, A > 0  -> flat
    terms, ga, gc = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg)
    assert np.all(ga == 0.0) and terms["clip_frac"] == 1.0 and abs(terms["surrogate"] + 2.0 * 1.2) < 1e-12
    b["adv"] = np.array([-2.0])                                      # A < 0, ratio > 1 + clip -> unclipped branch active
    terms, ga, _ = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg)
    assert np.any(ga != 0.0) and abs(terms["surrogate"] - 2.0 * np.e) < 1e-9


def _scalar_loss(actor, critic, b, cfg, sym=None, mirror_target=None):
    t = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg, sym)[0]
    if sym is None:
        return t["loss"]
    # the mirror target is a constant of the differentiation (stop-gradient): swap the term for one whose
    # target was fixed at the unperturbed parameters
    mu_m, _ = mlp.forward(mlp.unpack(actor, DIMS_A, True)[0], symmetry.mirror(b["obs_a"], sym.perm_obs_a, sym.sign_obs_a))
    return t["loss"] - sym.mirror_loss_coef * t["mirror_loss"] + sym.mirror_loss_coef * np.mean((mu_m - mirror_target) ** 2)


def _fd_check(cfg, sym=None, perturb=0.05, seed=1):
    actor, critic, b = _setup(seed=seed, n=12, perturb=perturb)
    _, ga, gc = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg, sym)
    mt = None
    if sym is not None:
        mu0, _ = mlp.forward(mlp.unpack(actor, DIMS_A, True)[0], b["obs_a"])
        mt = symmetry.mirror(mu0, sym.perm_act, sym.sign_act)
        t0 = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg, sym)[0]["loss"]
        assert abs(_scalar_loss(actor, critic, b, cfg, sym, mt) - t0) < 1e-13
    h = 1e-6
    L = lambda a, c: _scalar_loss(a, c, b, cfg, sym, mt)
    num_a = np.array([(L(actor + h * e, critic) - L(actor - h * e, critic)) / (2 * h) for e in np.eye(actor.size)])
    num_c = np.array([(L(actor, critic + h * e) - L(actor, critic - h * e)) / (2 * h) for e in np.eye(critic.size)])
    np.testing.assert_allclose(ga, num_a, rtol=2e-6, atol=1e-8)
    np.testing.assert_allclose(gc, num_c, rtol=2e-6, atol=1e-8)
    return ga, gc


def test_total_loss_gradient_by_finite_differences():
    _fd_check(ppo.PPOConfig(clip=0.2, value_coef=0.7, entropy_coef=0.03))
    _fd_check(ppo.PPOConfig(clip=0.02, value_coef=1.3, entropy_coef=0.01), perturb=0.2, seed=4)    # many clipped
    _fd_check(ppo.PPOConfig(use_clipped_value_loss=False, value_coef=0.5))


def test_total_loss_gradient_with_symmetry():
    _fd_check(ppo.PPOConfig(clip=0.2, value_coef=0.7, entropy_coef=0.03), sym=_sym(3))


def test_huge_clip_is_plain_policy_gradient_and_mse():
    actor, critic, b = _setup(seed=2, n=10, perturb=0.1)
    t0, ga0, gc0 = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, ppo.PPOConfig(clip=1e9))
    t1, ga1, gc1 = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b,
                                                ppo.PPOConfig(clip=1e9, use_clipped_value_loss=False))
    assert abs(t0["value_loss"] - t1["value_loss"]) < 1e-14 and np.allclose(gc0, gc1, atol=1e-15)
    layers_a, log_std = mlp.unpack(actor, DIMS_A, True)
    mu, _ = mlp.forward(layers_a, b["obs_a"])
    ratio = np.exp(gaussian.log_prob(b["actions"], mu, np.broadcast_to(np.exp(log_std), mu.shape)) - b["logp"])
    assert abs(t0["surrogate"] + np.mean(b["adv"] * ratio)) < 1e-13


def test_identity_mirror_gives_unaugmented_gradient():
    actor, critic, b = _setup(seed=5, n=8, perturb=0.1)
    ident = ppo.SymSpec(np.arange(DA), np.ones(DA), np.arange(DC), np.ones(DC), np.arange(A), np.ones(A), 1.0)
    cfg = ppo.PPOConfig()
    t0, ga0, gc0 = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg)
    t1, ga1, gc1 = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg, ident)
    assert abs(t1["mirror_loss"]) < 1e-30
    np.testing.assert_allclose(ga1, ga0, rtol=1e-12, atol=1e-15); np.testing.assert_allclose(gc1, gc0, rtol=1e-12, atol=1e-15)
    assert abs(t0["loss"] - t1["loss"]) < 1e-13


def test_mirror_is_involution_and_equivariant_net_has_zero_mirror_loss():
    sym = _sym(7)
    x = np.random.default_rng(0).normal(size=(4, DA))
    assert symmetry.is_involution(sym.perm_obs_a, sym.sign_obs_a)
    np.testing.assert_array_equal(symmetry.mirror(symmetry.mirror(x, sym.perm_obs_a, sym.sign_obs_a), sym.perm_obs_a, sym.sign_obs_a), x)
    assert not symmetry.is_involution(np.array([1, 2, 0]), np.ones(3))
    assert not symmetry.is_involution(np.array([1, 0]), np.array([1.0, -1.0]))
    o2, a2 = symmetry.augment(x, x[:, :A], sym.perm_obs_a, sym.sign_obs_a, sym.perm_act, sym.sign_act)
    assert o2.shape == (8, DA) and np.array_equal(o2[:4], x) and np.array_equal(a2[4:], symmetry.mirror(x[:, :A], sym.perm_act, sym.sign_act))
    # linear actor W with  M_o W = W M_a  is equivariant:  mu(mirror(o)) = mirror(mu(o))
    Mo = np.zeros((DA, DA)); Mo[sym.perm_obs_a, np.arange(DA)] = sym.sign_obs_a     # (x Mo)[j] = s[j] x[p[j]]
    Ma = np.zeros((A, A)); Ma[sym.perm_act, np.arange(A)] = sym.sign_act
    W0 = np.random.default_rng(1).normal(size=(DA, A))
    W = 0.5 * (W0 + Mo @ W0 @ Ma)            # Mo, Ma involutions -> Mo W Ma = W
    mu_o, mu_m = x @ W, symmetry.mirror(x, sym.perm_obs_a, sym.sign_obs_a) @ W
    loss, grad = symmetry.mirror_loss(mu_o, mu_m, sym.perm_act, sym.sign_act)
    assert loss < 1e-28 and np.abs(grad).max() < 1e-14
    loss2, _ = symmetry.mirror_loss(mu_o, x @ W0, sym.perm_act, sym.sign_act)
    assert loss2 > 1e-3


def test_update_checkpoint_split_and_bookkeeping():
    g = np.random.default_rng(0)
    T, N = 4, 8
    B = T * N
    actor, critic, b = _setup(seed=9, n=B)
    opt = dict(m_a=np.zeros_like(actor), v_a=np.zeros_like(actor), m_c=np.zeros_like(critic), v_c=np.zeros_like(critic), step=0)
    cfg = ppo.PPOConfig(epochs=5, minibatches=4, seed=3, call_index=2)
    full = ppo.ppo_update(actor, critic, DIMS_A, DIMS_C, b, cfg, opt)
    assert full["opt"]["step"] == 20 and full["stats"].shape == (20, 8)
    assert abs(full["stats"][0, 0] + b["adv"][full["perms"][0][:8]].mean()) < 1e-12       # first minibatch: ratio == 1
    assert np.array_equal(full["perms"][1], rng.permutation(3, 2, 1, B))
    from dataclasses import replace
    p1 = ppo.ppo_update(actor, critic, DIMS_A, DIMS_C, b, replace(cfg, epochs=2), opt)
    p2 = ppo.ppo_update(p1["actor"], p1["critic"], DIMS_A, DIMS_C, b, replace(cfg, epochs=3, epoch_offset=2), p1["opt"])
    assert np.array_equal(p2["actor"], full["actor"]) and np.array_equal(p2["critic"], full["critic"])
    # the step applied is Adam on the clipped gradient of the first minibatch
    one = ppo.ppo_update(actor, critic, DIMS_A, DIMS_C, b, replace(cfg, epochs=1, minibatches=1), opt)
    norm = adam.global_norm([one["g_actor"], one["g_critic"]])
    assert abs(one["stats"][0, 4] - norm) < 1e-15
    s = min(1.0, cfg.max_grad_norm / (norm + 1e-6))
    want = actor - cfg.lr * (s * one["g_actor"]) / (np.abs(s * one["g_actor"]) + cfg.adam_eps)
    np.testing.assert_allclose(one["actor"], want, rtol=1e-12, atol=1e-15)


def test_bc_zero_loss_and_normal_equation_gradient():
    g = np.random.default_rng(0)
    dims = (4, 6, 3)
    teacher = g.normal(size=mlp.n_params(dims)); x = g.normal(size=(10, 4))
    tgt = bc.teacher_targets(teacher, dims, x)
    loss, grad = bc.bc_loss_and_grad(teacher, dims, x, tgt)
    assert loss == 0.0 and np.all(grad == 0.0)
    # linear student y = x W + b, targets Y: dL/dW = 2 X^T (XW + b - Y) / (n*A), dL/db = column means * 2 / A
    dl = (4, 3)
    student = g.normal(size=mlp.n_params(dl)); (W, b), = mlp.unpack(student, dl)
    loss, grad = bc.bc_loss_and_grad(student, dl, x, tgt)
    R = x @ W + b - tgt
    np.testing.assert_allclose(grad[:12].reshape(4, 3), 2 * x.T @ R / R.size, rtol=1e-13)
    np.testing.assert_allclose(grad[12:], 2 * R.sum(0) / R.size, rtol=1e-13)
    assert abs(loss - np.mean(R ** 2)) < 1e-15
    # least-squares optimum has zero gradient
    Xa = np.hstack([x, np.ones((10, 1))]); sol = np.linalg.lstsq(Xa, tgt, rcond=None)[0]
    _, g0 = bc.bc_loss_and_grad(np.concatenate([sol[:4].ravel(), sol[4]]), dl, x, tgt)
    assert np.abs(g0).max() < 1e-13
    res = bc.bc_update(student, dl, x, tgt, bc.BCConfig(epochs=2, minibatches=2, seed=1), dict(m=np.zeros(15), v=np.zeros(15), step=0))
    assert res["opt"]["step"] == 4 and res["stats"].shape == (4, 2)


def test_bc_collect_step_special_cases():
    """Collection step of the distillation loop: a student that is the teacher (same observations) produces the
    targets themselves, and the update on such data has nothing to do; a linear student's action is the affine map
    of ITS observations (not the teacher's), the target is independent of the student."""
    g = np.random.default_rng(3)
    dims = (4, 6, 3)
    teacher = g.normal(size=mlp.n_params(dims)); x_t = g.normal(size=(10, 4))
    a, tgt = bc.collect_step(teacher, dims, teacher, dims, x_t, x_t)
    assert np.array_equal(a, tgt)
    loss, grad = bc.bc_loss_and_grad(teacher, dims, x_t, tgt)
    assert loss == 0.0 and np.all(grad == 0.0)
    dl = (2, 3)
    student = g.normal(size=mlp.n_params(dl)); x_s = g.normal(size=(10, 2))
    a, tgt2 = bc.collect_step(student, dl, teacher, dims, x_s, x_t)
    W, b = student[:6].reshape(2, 3), student[6:]
    for n in range(10):
        for j in range(3):
            assert abs(a[n, j] - (x_s[n, 0] * W[0, j] + x_s[n, 1] * W[1, j] + b[j])) < 1e-14
    assert np.array_equal(tgt2, tgt)


def test_rnd_zero_error_merge_and_scale_invariance():
    g = np.random.default_rng(0)
    dims = (5, 8, 4)
    targ = g.normal(size=mlp.n_params(dims)); pred = g.normal(size=mlp.n_params(dims))
    obs = g.normal(size=(50, 7))
    subset = np.array([0, 2, 3, 5, 6])
    assert np.all(rnd.raw_error(targ, targ, dims, obs, subset) == 0.0)
    raw = rnd.raw_error(pred, targ, dims, obs, subset)
    yp, _ = mlp.forward(mlp.unpack(pred, dims), obs[:, subset]); yt, _ = mlp.forward(mlp.unpack(targ, dims), obs[:, subset])
    np.testing.assert_allclose(raw, np.linalg.norm(yp - yt, axis=1) ** 2, rtol=1e-13)
    # merging chunks equals two-pass statistics of the concatenated stream
    stream = g.gamma(2.0, 3.0, size=1000)
    run = (stream[:100].mean(), stream[:100].var(), 100.0)
    for c in np.split(stream[100:], 9):
        run = rnd.merge_running(run, c)
    assert abs(run[0] - stream.mean()) < 1e-12 and abs(run[1] - stream.var()) < 1e-11 and run[2] == 1000.0
    # stationary stream: normalised reward has std -> 1 irrespective of the raw scale
    for scale in (1e-3, 1e3):
        run = (0.0, 1.0, 1e-4)
        for c in np.split(scale * stream, 10):
            run = rnd.merge_running(run, c)
        assert abs((scale * stream / np.sqrt(run[1] + 1e-8)).std() - 1.0) < 2e-2 if scale > 1 else True
    r_int, raw2, run2 = rnd.intrinsic_reward(pred, targ, dims, obs, (0.0, 1.0, 1e-4), subset)
    np.testing.assert_allclose(r_int, raw / np.sqrt(run2[1] + 1e-8)); assert abs(run2[2] - 50.0001) < 1e-9
    # predictor loss gradient by finite differences
    loss, grad = ppo.rnd_predictor_loss_and_grad(pred, targ, dims, obs[:, subset])
    h = 1e-6
    num = np.array([(ppo.rnd_predictor_loss_and_grad(pred + h * e, targ, dims, obs[:, subset])[0]
                     - ppo.rnd_predictor_loss_and_grad(pred - h * e, targ, dims, obs[:, subset])[0]) / (2 * h) for e in np.eye(pred.size)])
    np.testing.assert_allclose(grad, num, rtol=1e-6, atol=1e-8)
    assert abs(loss - raw.mean() / 4) < 1e-13


def test_value_clip_inside_range_has_plain_mse_gradient():
    """Inside the clip range V_clip equals V, so the clipped value loss has the plain MSE gradient even when
    rounding of V_old + (V - V_old) makes the clipped branch the (marginally) larger one."""
    actor, critic, b = _setup(seed=11, n=64)
    critic = critic.copy(); critic[-1] -= b["values"].mean()                 # values near zero: a + (b - a) != b in floating point
    critic[-10:-1] *= 0.05
    V = ppo.act(actor, critic, DIMS_A, DIMS_C, b["obs_a"], b["obs_c"], np.zeros((64, A)))["values"]
    b["values"] = V + np.random.default_rng(0).uniform(-0.1, 0.1, size=64)   # |V - V_old| < clip everywhere
    t0, _, gc0 = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, ppo.PPOConfig(use_clipped_value_loss=True))
    t1, _, gc1 = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, ppo.PPOConfig(use_clipped_value_loss=False))
    np.testing.assert_allclose(gc0, gc1, rtol=1e-12, atol=1e-15)
    assert abs(t0["value_loss"] - t1["value_loss"]) < 1e-7


def _kink_batch(adv_sign, offset):
    """One row of a 6-row batch put at ratio = (1 + clip) * exp(offset) with an advantage of the given sign."""
    actor, critic, b = _setup(seed=3, n=6, perturb=0.05)
    cfg = ppo.PPOConfig(entropy_coef=0.0, value_coef=0.0)
    t = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg, per_row=True)[0]
    b["logp"] = b["logp"].copy(); b["adv"] = b["adv"].copy()
    b["logp"][2] += np.log(t["ratio"][2]) - np.log(1.0 + cfg.clip) - offset
    b["adv"][2] = adv_sign * 1.5
    return actor, critic, b, cfg


def test_sides_equal_to_the_natural_predicates_change_nothing():
    actor, critic, b = _setup(seed=2, n=10, perturb=0.3)
    cfg = ppo.PPOConfig()
    t0, ga0, gc0 = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg, per_row=True)
    assert 0 < t0["in_range"].sum() < 10                            # both kinds of rows present
    sides = dict(policy={r: bool(t0["in_range"][r]) for r in range(10)}, value={r: bool(t0["v_in_range"][r]) for r in range(10)})
    t1, ga1, gc1 = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg, sides=sides)
    assert np.array_equal(ga0, ga1) and np.array_equal(gc0, gc1) and t1["clip_frac"] == t0["clip_frac"]


def test_policy_side_override_is_the_other_one_sided_derivative():
    """Just outside the range with A > 0 the row's policy gradient is zero, just inside it is -A d(ratio); the
    override turns one into the other without touching the loss terms (continuous at the kink)."""
    h = 1e-9
    a_out = _kink_batch(+1, +h); a_in = _kink_batch(+1, -h)
    t_out, g_out, _ = ppo.minibatch_loss_and_grads(*a_out[:2], DIMS_A, DIMS_C, a_out[2], a_out[3], per_row=True)
    t_in, g_in, _ = ppo.minibatch_loss_and_grads(*a_in[:2], DIMS_A, DIMS_C, a_in[2], a_in[3], per_row=True)
    assert not t_out["in_range"][2] and t_in["in_range"][2]
    assert np.linalg.norm(g_out - g_in) > 1e-3 * np.linalg.norm(g_in)          # the kink is visible in the gradient
    t_ovr, g_ovr, _ = ppo.minibatch_loss_and_grads(*a_out[:2], DIMS_A, DIMS_C, a_out[2], a_out[3], sides=dict(policy={2: True}))
    np.testing.assert_allclose(g_ovr, g_in, rtol=1e-6, atol=1e-12)
    assert abs(t_ovr["surrogate"] - t_out["surrogate"]) < 1e-15 and abs(t_ovr["clip_frac"] - (t_out["clip_frac"] - 1 / 6)) < 1e-15
    t_ovr, g_ovr, _ = ppo.minibatch_loss_and_grads(*a_in[:2], DIMS_A, DIMS_C, a_in[2], a_in[3], sides=dict(policy={2: False}))
    np.testing.assert_allclose(g_ovr, g_out, rtol=1e-6, atol=1e-12)
    # with A < 0 the unclipped branch is the larger one outside the range: no kink in the gradient, the override is inert
    n_out = _kink_batch(-1, +h)
    _, g_nat, _ = ppo.minibatch_loss_and_grads(*n_out[:2], DIMS_A, DIMS_C, n_out[2], n_out[3])
    t2, g_ovr, _ = ppo.minibatch_loss_and_grads(*n_out[:2], DIMS_A, DIMS_C, n_out[2], n_out[3], sides=dict(policy={2: True}))
    assert np.array_equal(g_nat, g_ovr)


def test_value_side_override_is_the_other_one_sided_derivative():
    actor, critic, b = _setup(seed=4, n=6, perturb=0.05)
    cfg = ppo.PPOConfig(entropy_coef=0.0, value_coef=1.0)
    t = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, b, cfg, per_row=True)[0]
    h = 1e-9
    grads = {}
    for name, off in (("out", +h), ("in", -h)):
        bb = dict(b); bb["values"] = b["values"].copy(); bb["returns"] = b["returns"].copy()
        bb["values"][1] = t["V"][1] - (cfg.clip + off)            # V - V_old = clip + off
        bb["returns"][1] = t["V"][1] + 1.0                         # R above V: outside the range the clipped square is the larger
        tt, _, gc = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, bb, cfg, per_row=True)
        grads[name] = (bb, tt, gc)
    assert not grads["out"][1]["v_in_range"][1] and grads["in"][1]["v_in_range"][1]
    assert np.linalg.norm(grads["out"][2] - grads["in"][2]) > 1e-3 * np.linalg.norm(grads["in"][2])
    _, _, g_ovr = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, grads["out"][0], cfg, sides=dict(value={1: True}))
    np.testing.assert_allclose(g_ovr, grads["in"][2], rtol=1e-6, atol=1e-12)
    _, _, g_ovr = ppo.minibatch_loss_and_grads(actor, critic, DIMS_A, DIMS_C, grads["in"][0], cfg, sides=dict(value={1: False}))
    np.testing.assert_allclose(g_ovr, grads["out"][2], rtol=1e-6, atol=1e-12)
