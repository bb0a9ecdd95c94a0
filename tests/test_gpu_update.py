"""GPU parity of the PPO and BC updates against the fp64 oracle: loss terms, gradients, post-update parameters."""
import ctypes as C
from dataclasses import replace
import numpy as np
import pytest
import torch

from oracle import ppo as oppo, bc as obc, mlp as omlp
from workloads import WORKLOADS, make_inputs
from gpu_util import dev, host, rel_l2, oracle_rollout, flat_rollout, oracle_cfg, f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rx():
    import paper_2509_10771_amd as m
    m.rslx_device_check()
    return m


def _layer_slices(dims, log_std):
    out, o = [], 0
    for l, (i, j) in enumerate(zip(dims[:-1], dims[1:])):
        out.append(("W%d" % l, slice(o, o + i * j))); o += i * j
        out.append(("b%d" % l, slice(o, o + j))); o += j
    if log_std:
        out.append(("log_std", slice(o, o + dims[-1])))
    return out


def _check_vec(name, dims, log_std, got, ref, tol, floor=0.0):
    for nm, sl in _layer_slices(dims, log_std):
        r = np.asarray(ref[sl], np.float64)
        err = np.linalg.norm(np.asarray(got[sl], np.float64) - r)
        assert err <= tol * max(np.linalg.norm(r), floor), (name, nm, err, np.linalg.norm(r))


def run_ppo(rx, w, epochs, sym_on=False, rnd_on=False, seed=3, call_index=1, epoch_offset=0, state=None):
    inp = make_inputs(w)
    ro = oracle_rollout(w, inp)
    flat = flat_rollout(w, inp, ro)
    ocfg = replace(oracle_cfg(w, epochs, seed, call_index), epoch_offset=epoch_offset)
    na, nc = inp["actor"].size, inp["critic"].size
    osym = None
    if sym_on:
        osym = oppo.SymSpec(inp["perm_obs"], inp["sign_obs"], inp["perm_obs"], inp["sign_obs"], inp["perm_act"],
                            inp["sign_act"], f32(w.mirror_loss_coef))
    opt0 = dict(m_a=np.zeros(na), v_a=np.zeros(na), m_c=np.zeros(nc), v_c=np.zeros(nc), step=0)
    ornd = None
    if rnd_on:
        npred = inp["rnd_predictor"].size
        ornd = dict(pred=inp["rnd_predictor"], targ=inp["rnd_target"], dims=w.dims_rnd, subset=None, m=np.zeros(npred),
                    v=np.zeros(npred), step=0, lr=f32(w.lr))
    ref = oppo.ppo_update(inp["actor"], inp["critic"], w.dims_actor, w.dims_critic, flat, ocfg, opt0, osym, ornd)

    actor = rx.Mlp(w.dims_actor, dev(inp["actor"]), trainable=True, has_log_std=True)
    critic = rx.Mlp(w.dims_critic, dev(inp["critic"]), trainable=True)
    d_obs = dev(flat["obs_a"])
    rollout = rx.Rollout(w.T, w.N, d_obs, d_obs, dev(flat["actions"]), dev(flat["logp"]), dev(flat["values"]),
                         dev(flat["mu"]), dev(flat["sigma"]), dev(flat["adv"]), dev(flat["returns"]))
    cfg = rx.PpoCfg(clip=w.clip, value_coef=w.value_coef, entropy_coef=w.entropy_coef, max_grad_norm=w.max_grad_norm,
                    lr=w.lr, epochs=epochs, minibatches=w.minibatches, seed=seed, call_index=call_index, epoch_offset=epoch_offset)
    sym = rx.Sym(inp["perm_obs"], inp["sign_obs"], inp["perm_obs"], inp["sign_obs"], inp["perm_act"], inp["sign_act"],
                 w.mirror_loss_coef) if sym_on else None
    rnd = None
    if rnd_on:
        rnd = rx.RndTrain(rx.Mlp(w.dims_rnd, dev(inp["rnd_target"])), rx.Mlp(w.dims_rnd, dev(inp["rnd_predictor"]), trainable=True), lr=w.lr)
    stats = torch.zeros(epochs * w.minibatches, rx.NSTATS, device="cuda")
    ws = rx.workspace(rx.rslx_ppo_update_workspace_bytes(actor, critic, rollout, cfg, sym, rnd))
    step = C.c_int64(0)
    rx.rslx_ppo_update(actor, critic, rollout, cfg, sym, rnd, step, stats, ws)
    torch.cuda.synchronize()
    return dict(ref=ref, actor=actor, critic=critic, stats=host(stats), step=step.value, rnd=rnd, inp=inp)


def check_ppo(w, res, epochs, rnd_on=False):
    ref = res["ref"]
    assert res["step"] == epochs * w.minibatches == ref["opt"]["step"]
    got, want = res["stats"], ref["stats"]
    for col in range(8):
        err = np.abs(got[:, col] - want[:, col])
        assert np.all(err <= 1e-4 * np.maximum(np.abs(want[:, col]), 1e-3)), (col, got[:, col], want[:, col])
    _check_vec("g_actor", w.dims_actor, True, host(res["actor"].grads), ref["g_actor"], 1e-4)
    _check_vec("g_critic", w.dims_critic, False, host(res["critic"].grads), ref["g_critic"], 1e-4)
    assert rel_l2(host(res["actor"].params), ref["actor"]) <= 1e-4
    assert rel_l2(host(res["critic"].params), ref["critic"]) <= 1e-4
    # the applied update itself (Adam turns tiny gradient entries into +-lr steps, hence the looser bound)
    d_got = host(res["actor"].params).astype(np.float64) - res["inp"]["actor"]
    d_ref = ref["actor"] - res["inp"]["actor"]
    assert rel_l2(d_got, d_ref) <= 2e-2
    np.testing.assert_allclose(host(res["actor"].adam_m), ref["opt"]["m_a"], rtol=0, atol=1e-4 * np.abs(ref["opt"]["m_a"]).max())
    if rnd_on:
        assert rel_l2(host(res["rnd"].predictor.params), ref["rnd"]["pred"]) <= 1e-4
        _check_vec("g_pred", w.dims_rnd, False, host(res["rnd"].predictor.grads), ref["rnd"]["g"], 1e-4)
        assert res["rnd"].step.value == ref["rnd"]["step"]


def test_ppo_tiny_one_epoch(rx):
    w = WORKLOADS["tiny"]
    check_ppo(w, run_ppo(rx, w, 1), 1)


def test_ppo_flat_ragged_one_epoch(rx):
    w = WORKLOADS["flat"].scaled(250)        # mb = 1500 rows: 11 full 128-row tiles and a 92-row tail
    check_ppo(w, run_ppo(rx, w, 1), 1)


def test_ppo_rough_symmetry_one_epoch(rx):
    w = WORKLOADS["rough"].scaled(125)
    check_ppo(w, run_ppo(rx, w, 1, sym_on=True), 1)


def test_ppo_curiosity_rnd_one_epoch(rx):
    w = replace(WORKLOADS["curiosity"].scaled(336), minibatches=8)
    check_ppo(w, run_ppo(rx, w, 1, rnd_on=True), 1, rnd_on=True)


def test_ppo_five_epoch_drift_is_bounded(rx):
    w = WORKLOADS["tiny"]
    res = run_ppo(rx, w, 5)
    ref = res["ref"]
    assert rel_l2(host(res["actor"].params), ref["actor"]) <= 1e-3
    assert rel_l2(host(res["critic"].params), ref["critic"]) <= 1e-3
    assert np.all(np.abs(res["stats"][:, :3] - ref["stats"][:, :3]) <= 5e-3 * np.maximum(np.abs(ref["stats"][:, :3]), 1e-2))


def test_ppo_resume_with_epoch_offset(rx):
    w = WORKLOADS["tiny"]
    full = run_ppo(rx, w, 2)
    a = run_ppo(rx, w, 1)
    # second call continues from the first one's state with epoch_offset = 1
    inp = a["inp"]
    ro = oracle_rollout(w, inp); flat = flat_rollout(w, inp, ro)
    d_obs = dev(flat["obs_a"])
    rollout = rx.Rollout(w.T, w.N, d_obs, d_obs, dev(flat["actions"]), dev(flat["logp"]), dev(flat["values"]),
                         dev(flat["mu"]), dev(flat["sigma"]), dev(flat["adv"]), dev(flat["returns"]))
    cfg = rx.PpoCfg(clip=w.clip, value_coef=w.value_coef, entropy_coef=w.entropy_coef, max_grad_norm=w.max_grad_norm,
                    lr=w.lr, epochs=1, minibatches=w.minibatches, seed=3, call_index=1, epoch_offset=1)
    stats = torch.zeros(w.minibatches, rx.NSTATS, device="cuda")
    ws = rx.workspace(rx.rslx_ppo_update_workspace_bytes(a["actor"], a["critic"], rollout, cfg))
    step = C.c_int64(a["step"])
    rx.rslx_ppo_update(a["actor"], a["critic"], rollout, cfg, None, None, step, stats, ws)
    torch.cuda.synchronize()
    assert step.value == full["step"]
    assert torch.equal(a["actor"].params, full["actor"].params) and torch.equal(a["critic"].params, full["critic"].params)


@pytest.mark.parametrize("name,kw", [("flat", {}), ("rough", {"sym_on": True})])
def test_ppo_full_size_one_epoch(rx, name, kw):
    w = WORKLOADS[name]
    check_ppo(w, run_ppo(rx, w, 1, **kw), 1)


def run_bc(rx, w, epochs, clip=0.0):
    inp = make_inputs(w)
    B = w.B
    obs_t = inp["obs"][:w.T].reshape(B, -1); obs_s = inp["obs_student"].reshape(B, -1)
    tgt = obc.teacher_targets(inp["teacher"], w.dims_actor, obs_t)
    ns = inp["student"].size
    ocfg = obc.BCConfig(lr=f32(w.lr), beta1=f32(0.9), beta2=f32(0.999), adam_eps=f32(1e-8), epochs=epochs,
                        minibatches=w.minibatches, max_grad_norm=f32(clip), seed=5, call_index=2)
    ref = obc.bc_update(inp["student"], w.dims_student, obs_s, tgt.astype(np.float32), ocfg, dict(m=np.zeros(ns), v=np.zeros(ns), step=0))
    student = rx.Mlp(w.dims_student, dev(inp["student"]), trainable=True)
    teacher = rx.Mlp(w.dims_actor, dev(inp["teacher"]))
    cfg = rx.BcCfg(lr=w.lr, epochs=epochs, minibatches=w.minibatches, max_grad_norm=clip, seed=5, call_index=2)
    stats = torch.zeros(epochs * w.minibatches, rx.NSTATS, device="cuda")
    ws = rx.workspace(rx.rslx_bc_update_workspace_bytes(student, teacher, B, cfg))
    step = C.c_int64(0)
    rx.rslx_bc_update(student, teacher, dev(obs_s), dev(obs_t), None, B, cfg, step, stats, ws)
    torch.cuda.synchronize()
    got = host(stats)
    assert step.value == epochs * w.minibatches
    assert np.all(np.abs(got[:, 0] - ref["stats"][:, 0]) <= 1e-4 * np.maximum(ref["stats"][:, 0], 1e-3))
    assert np.all(np.abs(got[:, 4] - ref["stats"][:, 1]) <= 1e-4 * np.maximum(ref["stats"][:, 1], 1e-3))
    _check_vec("g_student", w.dims_student, False, host(student.grads), ref["g"], 1e-4)
    assert rel_l2(host(student.params), ref["student"]) <= 1e-4
    # precomputed targets give the same result as the in-library teacher pass
    student2 = rx.Mlp(w.dims_student, dev(inp["student"]), trainable=True)
    step2 = C.c_int64(0)
    rx.rslx_bc_update(student2, None, dev(obs_s), None, dev(tgt.astype(np.float32)), B, cfg, step2, stats, ws)
    torch.cuda.synchronize()
    assert rel_l2(host(student2.params), ref["student"]) <= 1e-4


def test_bc_small(rx):
    run_bc(rx, WORKLOADS["distill"].scaled(125), 2)
    run_bc(rx, WORKLOADS["distill"].scaled(64), 1, clip=0.5)


def test_bc_full_size(rx):
    run_bc(rx, WORKLOADS["distill"], 1)
