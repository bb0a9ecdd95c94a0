"""GPU parity of the recurrent actor-critic (paper Sec. 3: hidden states managed across roll-outs, back-propagation
through time) against the fp64 oracle: act() with carried and reset states, and the column-wise PPO update, by
the same two comparisons as the feed-forward update (every optimiser step replayed from the oracle's state before
it; one free-running call)."""
import ctypes as C
from dataclasses import replace
import numpy as np
import pytest
import torch

from oracle import recurrent as orec, gae as ogae, rng as orng, ppo as oppo, gru as ogru
from workloads import WORKLOADS, make_inputs
from gpu_util import dev, host, rel_l2, f32, assert_elementwise
from test_gpu_update import _check_stats, _check_vec, _layer_slices, TOL

pytestmark = pytest.mark.gpu

SEED = 13


@pytest.fixture(scope="module")
def rx():
    import paper_2509_10771_amd as m
    m.rslx_device_check()
    return m


def _flat(inp, which):
    return np.concatenate([inp["mem_" + which], inp[which]])


def _cell(w):
    """(oracle module of the workload's cell, number of gates, packed state width)."""
    C = orec.CELLS[w.memory_cell]
    return C, C.GATES, C.state_width(w.memory_hidden)


def oracle_collect(w, inp):
    """Roll the oracle's recurrent act() over the T slabs (float32 storage of what the update consumes)."""
    T, N, A, H = w.T, w.N, w.A, w.memory_hidden
    actor, critic = _flat(inp, "actor"), _flat(inp, "critic")
    h_a, h_c, reset = inp["h_actor"].astype(np.float64), inp["h_critic"].astype(np.float64), inp["reset0"]
    acc = {k: [] for k in ("actions", "logp", "values", "mu", "sigma", "h_a", "h_c")}
    h0 = None
    for t in range(T):
        o = orec.act(actor, critic, w.Da, w.Dc, H, w.dims_actor, w.dims_critic, inp["obs"][t], inp["obs"][t], h_a, h_c, reset,
                     orng.act_noise(SEED, t, N, A), cell=w.memory_cell)
        if t == 0:
            h0 = (o["hin_a"], o["hin_c"])
        for k in acc:
            acc[k].append(o[k])
        h_a, h_c, reset = o["h_a"], o["h_c"], inp["dones"][t]
    last = orec.act(actor, critic, w.Da, w.Dc, H, w.dims_actor, w.dims_critic, inp["obs"][T], inp["obs"][T], h_a, h_c, reset,
                    np.zeros((N, A)), cell=w.memory_cell)["values"]
    c32 = lambda x: np.ascontiguousarray(np.asarray(x, np.float32))
    ro = {k: c32(np.stack(v)) for k, v in acc.items()}
    ro["h0_a"], ro["h0_c"], ro["last"] = c32(h0[0]), c32(h0[1]), c32(last)
    adv, ret = ogae.gae(inp["rewards"], ro["values"], ro["last"], inp["dones"], w.gamma, w.lam)
    ro["adv"], ro["returns"] = c32(ogae.normalize_advantages(adv)), c32(ret)
    return ro


def _nets(rx, w, actor_flat, critic_flat, opt=None):
    """(gru_a, mlp_a, gru_c, mlp_c) on slices of one flat device buffer per network and optimiser moment."""
    H = w.memory_hidden
    C, _, _ = _cell(w)
    cell_id = rx.CELL_LSTM if w.memory_cell == "lstm" else rx.CELL_GRU
    out = []
    for flat, D, dims, log_std, mk, vk in ((actor_flat, w.Da, w.dims_actor, True, "m_a", "v_a"),
                                           (critic_flat, w.Dc, w.dims_critic, False, "m_c", "v_c")):
        k = C.n_params(D, H)
        p = dev(flat, torch.float32)
        g = rx.Memory(cell_id, D, H, p[:k], trainable=True)
        m = rx.Mlp(dims, p[k:], trainable=True, has_log_std=log_std)
        if opt is not None:
            mm, vv = dev(opt[mk], torch.float32), dev(opt[vk], torch.float32)
            g.adam_m, g.adam_v, m.adam_m, m.adam_v = mm[:k], vv[:k], mm[k:], vv[k:]
        out += [g, m]
    return out


def _params(g, m):
    return np.concatenate([host(g.params), host(m.params)])


def _grads(g, m):
    return np.concatenate([host(g.grads), host(m.grads)])


@pytest.mark.parametrize("cell", ["gru", "lstm"])
@pytest.mark.parametrize("N", [64, 300])
def test_act_recurrent_matches_oracle(rx, N, cell):
    w = replace(WORKLOADS["recurrent"].scaled(N), memory_cell=cell)
    inp = make_inputs(w)
    ref = oracle_collect(w, inp)
    T, A, H = w.T, w.A, w.memory_hidden
    ga, ma, gc, mc = _nets(rx, w, _flat(inp, "actor"), _flat(inp, "critic"))
    h_a, h_c = dev(inp["h_actor"]), dev(inp["h_critic"])
    S = _cell(w)[2]
    h0_a, h0_c = torch.zeros(N, S, device="cuda"), torch.zeros(N, S, device="cuda")
    obs, dones = dev(inp["obs"]), dev(inp["dones"])
    reset = dev(inp["reset0"])
    assert inp["reset0"].sum() > 0 or N < 100
    out = {k: torch.empty(N, A, device="cuda") for k in ("actions", "mu", "sigma")}
    logp, values = torch.empty(N, device="cuda"), torch.empty(N, device="cuda")
    ws = rx.workspace(rx.rslx_act_recurrent_workspace_bytes(ga, ma, gc, mc, N))
    for t in range(T):
        eps = dev(orng.act_noise(SEED, t, N, A), torch.float32)
        rx.rslx_act_recurrent(ga, ma, gc, mc, obs[t], obs[t], N, h_a, h_c, reset if t == 0 else dones[t - 1],
                              h0_a if t == 0 else None, h0_c if t == 0 else None, SEED, t, eps, out["actions"], logp, values,
                              out["mu"], out["sigma"], 0, ws)
        torch.cuda.synchronize()
        for k in ("actions", "mu", "sigma"):
            assert rel_l2(host(out[k]), ref[k][t]) <= 2e-5, (t, k)
            assert_elementwise("%s[%d]" % (k, t), host(out[k]), ref[k][t])
        assert rel_l2(host(logp), ref["logp"][t]) <= 2e-5 and rel_l2(host(values), ref["values"][t]) <= 2e-5
        assert rel_l2(host(h_a), ref["h_a"][t]) <= 2e-5 and rel_l2(host(h_c), ref["h_c"][t]) <= 2e-5
        for nm, got_t, ref_t in (("logp", logp, ref["logp"][t]), ("values", values, ref["values"][t]), ("h_a", h_a, ref["h_a"][t]),
                                 ("h_c", h_c, ref["h_c"][t])):
            assert_elementwise("%s[%d]" % (nm, t), host(got_t), ref_t)
    assert rel_l2(host(h0_a), ref["h0_a"]) <= 1e-6 and rel_l2(host(h0_c), ref["h0_c"]) <= 1e-6
    # the bootstrap value leaves both states untouched
    before = (h_a.clone(), h_c.clone())
    last = torch.empty(N, device="cuda")
    rx.rslx_act_recurrent(None, None, gc, mc, None, obs[T], N, None, h_c, dones[T - 1], None, None, 0, 0, None, None, None, last,
                          None, None, rx.ACT_VALUES_ONLY, ws)
    torch.cuda.synchronize()
    assert rel_l2(host(last), ref["last"]) <= 2e-5
    assert torch.equal(h_a, before[0]) and torch.equal(h_c, before[1])
    # the GPU's own noise stream is the one rslx_act uses
    rx.rslx_act_recurrent(ga, ma, gc, mc, obs[0], obs[0], N, h_a, h_c, None, None, None, SEED, 5, None, out["actions"], logp, values,
                          out["mu"], out["sigma"], 0, ws)
    torch.cuda.synchronize()
    z = (host(out["actions"]) - host(out["mu"])) / host(out["sigma"])
    np.testing.assert_allclose(z, orng.act_noise(SEED, 5, N, A), rtol=0, atol=2e-4)


class RCase:
    def __init__(self, w, epochs, seed=3, call_index=1, perturb=0.0):
        self.w, self.epochs, self.seed, self.call_index = w, epochs, seed, call_index
        inp = self.inp = make_inputs(w)
        ro = self.ro = oracle_collect(w, inp)
        self.actor0, self.critic0 = _flat(inp, "actor").astype(np.float32), _flat(inp, "critic").astype(np.float32)
        if perturb:
            g = np.random.default_rng(5)
            self.actor0 = (self.actor0 + perturb * g.standard_normal(self.actor0.size) * np.abs(self.actor0).mean()).astype(np.float32)
            self.critic0 = (self.critic0 + perturb * g.standard_normal(self.critic0.size) * np.abs(self.critic0).mean()).astype(np.float32)
        self.oro = dict(obs_a=inp["obs"][:w.T], obs_c=inp["obs"][:w.T], dones=inp["dones"], h0_a=ro["h0_a"], h0_c=ro["h0_c"],
                        **{k: ro[k] for k in ("actions", "logp", "values", "mu", "sigma", "adv", "returns")})
        self.ocfg = oppo.PPOConfig(clip=f32(w.clip), value_coef=f32(w.value_coef), entropy_coef=f32(w.entropy_coef),
                                   max_grad_norm=f32(w.max_grad_norm), lr=f32(w.lr), beta1=f32(0.9), beta2=f32(0.999),
                                   adam_eps=f32(1e-8), epochs=epochs, minibatches=w.minibatches, seed=seed, call_index=call_index)
        na, nc = self.actor0.size, self.critic0.size
        opt0 = dict(m_a=np.zeros(na), v_a=np.zeros(na), m_c=np.zeros(nc), v_c=np.zeros(nc), step=0)
        self.ref = orec.ppo_update(self.actor0, self.critic0, w.Da, w.Dc, w.memory_hidden, w.dims_actor, w.dims_critic, self.oro,
                                   self.ocfg, opt0, record=True, cell=w.memory_cell)

    def gpu_rollout(self, rx, envs=None):
        o = self.oro if envs is None else {k: (v[envs] if k in ("h0_a", "h0_c") else v[:, envs]) for k, v in self.oro.items()}
        N = o["dones"].shape[1]
        d_obs = dev(o["obs_a"])
        ro = rx.Rollout(self.w.T, N, d_obs, d_obs, dev(o["actions"]), dev(o["logp"]), dev(o["values"]), dev(o["mu"]),
                        dev(o["sigma"]), dev(o["adv"]), dev(o["returns"]))
        return ro, dev(o["dones"]), dev(o["h0_a"]), dev(o["h0_c"])

    def gpu_cfg(self, rx, epochs, minibatches):
        w = self.w
        return rx.PpoCfg(clip=w.clip, value_coef=w.value_coef, entropy_coef=w.entropy_coef, max_grad_norm=w.max_grad_norm,
                         lr=w.lr, epochs=epochs, minibatches=minibatches, seed=self.seed, call_index=self.call_index)


def _call(rx, nets, ro_pack, cfg, n_rows, step0):
    ro, dones, h0a, h0c = ro_pack
    stats = torch.zeros(n_rows, rx.NSTATS, device="cuda")
    ws = rx.workspace(rx.rslx_ppo_update_recurrent_workspace_bytes(*nets, ro, cfg))
    step = C.c_int64(step0)
    rx.rslx_ppo_update_recurrent(*nets, ro, dones, h0a, h0c, cfg, step, stats, ws)
    torch.cuda.synchronize()
    return host(stats), step.value


def _layer_names(w, which):
    """Size of the memory part, which comes first in a network's flat vector."""
    return _cell(w)[0].n_params(w.Da if which == "actor" else w.Dc, w.memory_hidden)


def _check_net(name, w, which, got, ref, tol, elementwise=False):
    k = _layer_names(w, which)
    D, H = (w.Da if which == "actor" else w.Dc), w.memory_hidden
    o = 0
    G = _cell(w)[1]
    for nm, n in (("W_ih", D * G * H), ("b_ih", G * H), ("W_hh", H * G * H), ("b_hh", G * H)):
        r = np.asarray(ref[o:o + n], np.float64)
        err = np.linalg.norm(np.asarray(got[o:o + n], np.float64) - r)
        assert err <= tol * np.linalg.norm(r) + 1e-12, (name, nm, err, np.linalg.norm(r))
        if elementwise:
            assert_elementwise("%s %s" % (name, nm), got[o:o + n], r, tol)
        o += n
    dims = w.dims_actor if which == "actor" else w.dims_critic
    _check_vec(name, dims, which == "actor", got[k:], ref[k:], tol)
    if elementwise:
        for nm, sl in _layer_slices(dims, which == "actor"):
            assert_elementwise("%s %s" % (name, nm), got[k:][sl], np.asarray(ref[k:][sl], np.float64), tol)


def check_forced_steps(rx, case, steps=None, floor=1e-3):
    w, ref = case.w, case.ref
    for k, tr in enumerate(ref["trace"]):
        if steps is not None and k not in steps:
            continue
        b = tr["before"]
        nets = _nets(rx, w, b["actor"], b["critic"], b["opt"])
        stats, step = _call(rx, nets, case.gpu_rollout(rx, tr["envs"]), case.gpu_cfg(rx, 1, 1), 1, b["opt"]["step"])
        assert step == b["opt"]["step"] + 1
        _check_stats(stats[0], ref["stats"][k], TOL, floor=floor)
        _check_net("g_actor step %d" % k, w, "actor", _grads(nets[0], nets[1]), tr["g_actor"], TOL, elementwise=True)
        _check_net("g_critic step %d" % k, w, "critic", _grads(nets[2], nets[3]), tr["g_critic"], TOL, elementwise=True)
        _check_net("actor step %d" % k, w, "actor", _params(nets[0], nets[1]), tr["actor"], TOL)
        _check_net("critic step %d" % k, w, "critic", _params(nets[2], nets[3]), tr["critic"], TOL)


def check_free_running(rx, case, later_tol=2e-2, param_tol=None, floor=1e-3):
    w, ref = case.w, case.ref
    nets = _nets(rx, w, case.actor0, case.critic0)
    n = case.epochs * w.minibatches
    stats, step = _call(rx, nets, case.gpu_rollout(rx), case.gpu_cfg(rx, case.epochs, w.minibatches), n, 0)
    assert step == n == ref["opt"]["step"]
    _check_stats(stats[0], ref["stats"][0], TOL, floor=floor)
    _check_stats(stats, ref["stats"], later_tol, floor=max(floor, 1e-2))
    param_tol = TOL * max(1, case.epochs) if param_tol is None else param_tol
    assert rel_l2(_params(nets[0], nets[1]), ref["actor"]) <= param_tol
    assert rel_l2(_params(nets[2], nets[3]), ref["critic"]) <= param_tol
    return nets, stats


@pytest.mark.parametrize("cell", ["gru", "lstm"])
def test_recurrent_update_small(rx, cell):
    w = replace(WORKLOADS["recurrent"].scaled(64), hidden=(128, 128), memory_hidden=64, done_p=0.05, memory_cell=cell)
    case = RCase(w, 1)
    assert case.inp["dones"][:-1].sum() > 10
    check_forced_steps(rx, case)
    check_free_running(rx, case)


@pytest.mark.parametrize("cell", ["gru", "lstm"])
def test_recurrent_update_off_policy_start_odd_shapes(rx, cell):
    """Ragged everything: 35 environments per minibatch, widths that are no multiple of the tiles, the unfused loss path."""
    w = replace(WORKLOADS["recurrent"].scaled(140), T=9, Da=21, Dc=21, A=5, hidden=(72, 40), memory_hidden=44, done_p=0.08,
                memory_cell=cell)
    case = RCase(w, 1, perturb=0.2)
    assert case.ref["stats"][0, 5] > 0.01
    check_forced_steps(rx, case)
    check_free_running(rx, case)


def test_recurrent_update_action_vector_wider_than_the_fused_head(rx):
    """40 action components: past the widths of the fused loss head, inside the ABI's maximum of 64."""
    w = replace(WORKLOADS["recurrent"].scaled(48), T=6, A=40, hidden=(64, 64), memory_hidden=32, done_p=0.1)
    case = RCase(w, 1, perturb=0.2)
    check_forced_steps(rx, case)
    check_free_running(rx, case)


@pytest.mark.parametrize("cell", ["gru", "lstm"])
def test_recurrent_update_two_epochs(rx, cell):
    w = replace(WORKLOADS["recurrent"].scaled(128), hidden=(256, 128), memory_hidden=128, done_p=0.03, memory_cell=cell)
    case = RCase(w, 2)
    check_free_running(rx, case, later_tol=5e-2)


@pytest.mark.parametrize("name", ["recurrent", "recurrent_lstm"])
def test_recurrent_update_full_width(rx, name):
    """The benchmark's network shapes (256-wide memories, [512, 256, 128] MLPs) at 512 environments."""
    case = RCase(WORKLOADS[name].scaled(512), 1)
    check_forced_steps(rx, case, steps={0, 3})
    check_free_running(rx, case)


def test_recurrent_update_rejects_bad_shapes(rx):
    w = replace(WORKLOADS["recurrent"].scaled(30), hidden=(32, 32), memory_hidden=16)
    inp = make_inputs(w)
    nets = _nets(rx, w, _flat(inp, "actor"), _flat(inp, "critic"))
    z = lambda *s: torch.zeros(*s, device="cuda")
    ro = rx.Rollout(w.T, 30, z(w.T, 30, w.Da), z(w.T, 30, w.Da), z(w.T, 30, w.A), z(w.T, 30), z(w.T, 30), z(w.T, 30, w.A),
                    z(w.T, 30, w.A), z(w.T, 30), z(w.T, 30))
    with pytest.raises(rx.RslxError):      # 30 environments do not split into 4 minibatches
        rx.rslx_ppo_update_recurrent_workspace_bytes(*nets, ro, rx.PpoCfg(epochs=1, minibatches=4))
    bad = rx.Gru(w.Da, 16, nets[0].params, trainable=True)
    bad.hidden = 18
    with pytest.raises(rx.RslxError):      # memory width must be a multiple of 4 (and match the MLP input)
        rx.rslx_ppo_update_recurrent_workspace_bytes(bad, nets[1], nets[2], nets[3], ro, rx.PpoCfg(epochs=1, minibatches=3))


@pytest.mark.parametrize("cell", ["gru", "lstm"])
@pytest.mark.parametrize("T,N,M,done_p", [(1, 32, 4, 0.1), (5, 4, 4, 0.3), (6, 48, 2, 1.0), (6, 48, 2, 0.0)])
def test_recurrent_update_degenerate_shapes(rx, T, N, M, done_p, cell):
    """One-step roll-outs, one environment per minibatch, an episode end on every step (no state is ever carried:
    the memory acts as a feed-forward layer) and none at all."""
    w = replace(WORKLOADS["recurrent"].scaled(N), T=T, minibatches=M, hidden=(64, 32), memory_hidden=32, done_p=done_p,
                memory_cell=cell)
    case = RCase(w, 1, perturb=0.1)
    if done_p == 1.0:
        assert case.inp["dones"].all()
    # with 5 to 96 samples per minibatch the surrogate is a mean of a few O(1) terms of both signs and can come out
    # near zero; its fp32 rounding is relative to the terms, so the statistics are compared with a floor of 0.05
    check_forced_steps(rx, case, floor=5e-2)
    check_free_running(rx, case, floor=5e-2)


def test_recurrent_empty_calls_are_no_ops(rx):
    w = replace(WORKLOADS["recurrent"].scaled(16), hidden=(32, 32), memory_hidden=16)
    inp = make_inputs(w)
    ro = oracle_collect(w, inp)
    nets = _nets(rx, w, _flat(inp, "actor"), _flat(inp, "critic"))
    before = [host(n.params).copy() for n in nets]
    # zero environments in act
    rx.rslx_act_recurrent(nets[0], nets[1], nets[2], nets[3], dev(inp["obs"][0]), dev(inp["obs"][0]), 0, dev(inp["h_actor"]),
                          dev(inp["h_critic"]), None, None, None, SEED, 0, None, torch.zeros(1, device="cuda"),
                          torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda"),
                          torch.zeros(1, device="cuda"), 0, rx.workspace(256))
    # zero epochs in the update
    case_ro = dict(obs_a=inp["obs"][:w.T], dones=inp["dones"], h0_a=ro["h0_a"], h0_c=ro["h0_c"],
                   **{k: ro[k] for k in ("actions", "logp", "values", "mu", "sigma", "adv", "returns")})
    d_obs = dev(case_ro["obs_a"])
    g_ro = rx.Rollout(w.T, w.N, d_obs, d_obs, dev(case_ro["actions"]), dev(case_ro["logp"]), dev(case_ro["values"]),
                      dev(case_ro["mu"]), dev(case_ro["sigma"]), dev(case_ro["adv"]), dev(case_ro["returns"]))
    cfg = rx.PpoCfg(epochs=0, minibatches=4)
    stats = torch.zeros(1, rx.NSTATS, device="cuda")
    step = C.c_int64(3)
    ws = rx.workspace(rx.rslx_ppo_update_recurrent_workspace_bytes(*nets, g_ro, cfg))
    rx.rslx_ppo_update_recurrent(*nets, g_ro, dev(inp["dones"]), dev(ro["h0_a"]), dev(ro["h0_c"]), cfg, step, stats, ws)
    torch.cuda.synchronize()
    assert step.value == 3
    for n, b in zip(nets, before):
        assert np.array_equal(host(n.params), b)


@pytest.mark.parametrize("name", ["recurrent", "recurrent_lstm"])
def test_recurrent_update_full_size(rx, name):
    """The benchmark's configuration itself (4096 environments, minibatches of 1024 columns x 24 steps): the first and
    the last optimiser step of an epoch replayed from the oracle's state, and the collection loop's first steps."""
    case = RCase(WORKLOADS[name], 1)
    check_forced_steps(rx, case, steps={0, 3})
