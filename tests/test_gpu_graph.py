"""GPU tests of the replayable entry points (call-to-call counters in device memory) and of a whole training
iteration (T x act, value bootstrap, GAE, PPO update; paper Sec. 3) recorded once as a HIP graph and replayed.

  * rslx_act_dc / rslx_ppo_update_dc against the oracle (same bar as the host-counter entry points);
  * an eager loop on device counters against the same loop on host counters (identical noise and permutations;
    the Adam bias corrections come from the device's fp64 pow instead of the host's, so parameters may differ in
    the last bit);
  * graph replays against the eager device-counter loop, bit for bit, three replays in a row with eager library
    work and synchronisation between them.
"""
import ctypes as C
from dataclasses import replace
import numpy as np
import pytest
import torch

from oracle import ppo as oppo, rng as orng
from workloads import WORKLOADS, make_inputs
from gpu_util import dev, host, rel_l2, assert_elementwise
from test_gpu_update import Case, _nets, _check_stats, TOL

pytestmark = pytest.mark.gpu

SEED = 77


@pytest.fixture(scope="module")
def rx():
    import paper_2509_10771_amd as m
    m.rslx_device_check()
    return m


def test_act_dc_matches_oracle_at_the_counter_position(rx):
    w = WORKLOADS["tiny"]
    inp = make_inputs(w)
    N, A = w.N, w.A
    actor = rx.Mlp(w.dims_actor, dev(inp["actor"]), has_log_std=True)
    critic = rx.Mlp(w.dims_critic, dev(inp["critic"]))
    ws = rx.workspace(rx.rslx_act_workspace_bytes(actor, critic, N))
    ctr = rx.dev_counters(act_step=41)
    obs = dev(inp["obs"])
    out = {k: torch.empty(N, A, device="cuda") for k in ("actions", "mu", "sigma")}
    logp, values = torch.empty(N, device="cuda"), torch.empty(N, device="cuda")
    for k in range(3):
        rx.rslx_act_dc(actor, critic, obs[k], obs[k], N, SEED, ctr, None, out["actions"], logp, values, out["mu"],
                       out["sigma"], 0, ws)
        ref = oppo.act(inp["actor"], inp["critic"], w.dims_actor, w.dims_critic, inp["obs"][k], inp["obs"][k],
                       orng.act_noise(SEED, 41 + k, N, A))
        for name in ("actions", "mu", "sigma"):
            assert rel_l2(host(out[name]), ref[name]) <= 1e-5, (k, name)
            assert_elementwise(name, host(out[name]), ref[name])
        assert rel_l2(host(logp), ref["logp"]) <= 1e-5 and rel_l2(host(values), ref["values"]) <= 1e-5
        assert_elementwise("logp", host(logp), ref["logp"]); assert_elementwise("values", host(values), ref["values"])
    # the value bootstrap draws no noise and leaves the position where it is
    rx.rslx_act_dc(None, critic, None, obs[3], N, SEED, ctr, None, None, None, values, None, None, rx.ACT_VALUES_ONLY, ws)
    assert host(ctr).tolist() == [44, 0, 0, 0]


@pytest.mark.parametrize("name,N,kw", [("tiny", 64, {}), ("curiosity", 84, {"rnd_on": True})])
def test_ppo_update_dc_matches_oracle(rx, name, N, kw):
    """One whole update call on device counters against the oracle's trajectory (first step to 1e-4, final
    parameters to 1e-4 per epoch), and the counters it leaves behind."""
    w = WORKLOADS[name].scaled(N)
    if name == "curiosity":
        w = replace(w, minibatches=4)
    case = Case(w, 1, call_index=6, **kw)
    ref = case.ref
    a, c, rnd = _nets(rx, case, case.actor0, case.critic0)
    n = case.epochs * w.minibatches
    ro, cfg, sym = case.gpu_rollout(rx), case.gpu_cfg(rx, case.epochs, w.minibatches), case.gpu_sym(rx)
    cfg.c.call_index = 999                      # ignored by the device-counter entry point
    stats = torch.zeros(n, rx.NSTATS, device="cuda")
    ws = rx.workspace(rx.rslx_ppo_update_workspace_bytes(a, c, ro, cfg, sym, rnd))
    ctr = rx.dev_counters(call_index=6)
    rx.rslx_ppo_update_dc(a, c, ro, cfg, sym, rnd, ctr, stats, ws)
    torch.cuda.synchronize()
    _check_stats(host(stats)[0], ref["stats"][0], TOL)
    _check_stats(host(stats), ref["stats"], 2e-2, floor=1e-2)
    assert rel_l2(host(a.params), ref["actor"]) <= TOL and rel_l2(host(c.params), ref["critic"]) <= TOL
    if case.rnd_on:
        assert rel_l2(host(rnd.predictor.params), ref["rnd"]["pred"]) <= TOL
    assert host(ctr).tolist() == [0, 7, n, n if case.rnd_on else 0]


class Loop:
    """The training iteration on one set of device buffers, on host counters or on device counters."""

    def __init__(self, rx, w, inp, device_counters, start=(0, 0, 0, 0)):
        self.rx, self.w, self.dc = rx, w, device_counters
        T, N, A = w.T, w.N, w.A
        self.actor = rx.Mlp(w.dims_actor, dev(inp["actor"]), trainable=True, has_log_std=True)
        self.critic = rx.Mlp(w.dims_critic, dev(inp["critic"]), trainable=True)
        self.obs, self.rewards, self.dones = dev(inp["obs"]), dev(inp["rewards"]), dev(inp["dones"])
        self.actions, self.mu, self.sigma = (torch.zeros(T, N, A, device="cuda") for _ in range(3))
        self.logp, self.values, self.adv, self.ret = (torch.zeros(T, N, device="cuda") for _ in range(4))
        self.last = torch.zeros(N, device="cuda")
        self.rnd = None
        if w.rnd:
            self.rnd_t = rx.Mlp(w.dims_rnd, dev(inp["rnd_target"]))
            self.rnd_p = rx.Mlp(w.dims_rnd, dev(inp["rnd_predictor"]), trainable=True)
            self.rnd = rx.RndTrain(self.rnd_t, self.rnd_p, lr=w.lr, adam_step=start[3])
            self.running = dev(np.array([0.0, 1.0, 1e-4], np.float32))
            self.r_int = torch.zeros(N, device="cuda")
            self.rws = rx.workspace(rx.rslx_rnd_workspace_bytes(self.rnd_t, N))
            self.rew_work = torch.zeros_like(self.rewards)
        self.rollout = rx.Rollout(T, N, self.obs[:T], self.obs[:T], self.actions, self.logp, self.values, self.mu,
                                  self.sigma, self.adv, self.ret)
        self.cfg_kw = dict(clip=w.clip, value_coef=w.value_coef, entropy_coef=w.entropy_coef, max_grad_norm=w.max_grad_norm,
                           lr=w.lr, epochs=2, minibatches=w.minibatches, seed=SEED)
        self.stats = torch.zeros(2 * w.minibatches, rx.NSTATS, device="cuda")
        self.aws = rx.workspace(rx.rslx_act_workspace_bytes(self.actor, self.critic, N))
        self.gws = rx.workspace(rx.rslx_gae_workspace_bytes(T, N))
        self.uws = rx.workspace(rx.rslx_ppo_update_workspace_bytes(self.actor, self.critic, self.rollout,
                                                                   rx.PpoCfg(**self.cfg_kw), None, self.rnd))
        self.start = start
        self.act_step, self.call_index, self.adam_step = start[0], start[1], C.c_int64(start[2])
        self.ctr = rx.dev_counters(*start) if device_counters else None
        self.state = [t.clone() for t in self.state_tensors()]

    def state_tensors(self):
        ts = [self.actor.params, self.actor.adam_m, self.actor.adam_v, self.critic.params, self.critic.adam_m, self.critic.adam_v]
        if self.rnd is not None:
            ts += [self.rnd_p.params, self.rnd_p.adam_m, self.rnd_p.adam_v, self.running]
        if self.ctr is not None:
            ts.append(self.ctr)
        return ts

    def reset(self):
        for t, t0 in zip(self.state_tensors(), self.state):
            t.copy_(t0)

    def outputs(self):
        ts = [self.actions, self.mu, self.sigma, self.logp, self.values, self.last, self.adv, self.ret, self.stats,
              self.actor.params, self.critic.params, self.actor.adam_v]
        if self.rnd is not None:
            ts += [self.rnd_p.params, self.running]
        return ts

    def iterate(self):
        rx, w = self.rx, self.w
        T, N = w.T, w.N
        rew = self.rewards
        if w.rnd:
            self.rew_work.copy_(self.rewards)
            rew = self.rew_work
        for t in range(T):
            o = self.obs[t]
            outs = (self.actions[t], self.logp[t], self.values[t], self.mu[t], self.sigma[t])
            if self.dc:
                rx.rslx_act_dc(self.actor, self.critic, o, o, N, SEED, self.ctr, None, *outs, 0, self.aws)
            else:
                rx.rslx_act(self.actor, self.critic, o, o, N, SEED, self.act_step, None, *outs, 0, self.aws)
                self.act_step += 1
            if w.rnd:
                rx.rslx_rnd(self.rnd_t, self.rnd_p, o, N, w.Da, None, w.Da, self.running, w.rnd_weight, 1, self.r_int,
                            rew[t], self.rws)
        if self.dc:
            rx.rslx_act_dc(None, self.critic, None, self.obs[T], N, SEED, self.ctr, None, None, None, self.last, None,
                           None, rx.ACT_VALUES_ONLY, self.aws)
        else:
            rx.rslx_act(None, self.critic, None, self.obs[T], N, 0, 0, None, None, None, self.last, None, None,
                        rx.ACT_VALUES_ONLY, self.aws)
        rx.rslx_gae(rew, self.values, self.last, self.dones, None, T, N, w.gamma, w.lam, 1, self.adv, self.ret, self.gws)
        if self.dc:
            rx.rslx_ppo_update_dc(self.actor, self.critic, self.rollout, rx.PpoCfg(**self.cfg_kw), None, self.rnd, self.ctr,
                                  self.stats, self.uws)
        else:
            rx.rslx_ppo_update(self.actor, self.critic, self.rollout, rx.PpoCfg(call_index=self.call_index, **self.cfg_kw),
                               None, self.rnd, self.adam_step, self.stats, self.uws)
            self.call_index += 1


def _workload(name):
    if name == "tiny":
        return WORKLOADS["tiny"]
    return replace(WORKLOADS["curiosity"].scaled(96), minibatches=4)


@pytest.mark.parametrize("name", ["tiny", "curiosity"])
def test_device_counter_loop_matches_host_counter_loop(rx, name):
    w = _workload(name)
    inp = make_inputs(w)
    start = (5, 3, 7, 7)
    h, d = Loop(rx, w, inp, False, start), Loop(rx, w, inp, True, start)
    n = 2 * w.minibatches
    for it in range(2):
        h.iterate(); d.iterate()
        torch.cuda.synchronize()
        if it == 0:      # same parameters, same noise position: the rollout is identical
            assert torch.equal(h.actions, d.actions) and torch.equal(h.adv, d.adv)
        for th, td in zip(h.outputs(), d.outputs()):
            assert rel_l2(host(td), host(th)) <= 1e-5
        want = [5 + (it + 1) * w.T, 3 + it + 1, 7 + (it + 1) * n, 7 + (it + 1) * n if w.rnd else 7]
        assert host(d.ctr).tolist() == want
        assert [h.act_step, h.call_index, h.adam_step.value] == want[:3]


@pytest.mark.parametrize("name", ["tiny", "curiosity"])
def test_iteration_graph_replays_match_eager(rx, name):
    """One iteration recorded as a graph and replayed three times must give, replay by replay, exactly what the
    eager device-counter loop gives: noise, permutations and Adam step counts advance on the device."""
    w = _workload(name)
    inp = make_inputs(w)
    eager, rec = Loop(rx, w, inp, True), Loop(rx, w, inp, True)
    rec.iterate()                     # first-use set-up of the kernels happens outside the recording
    torch.cuda.synchronize()
    rec.reset()
    for t in rec.outputs()[:9]:
        t.zero_()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rec.iterate()
    torch.cuda.synchronize()
    assert host(rec.ctr).tolist() == [0, 0, 0, 0] and float(rec.stats.abs().sum()) == 0.0    # recording ran nothing
    n = 2 * w.minibatches
    for k in range(3):
        g.replay()
        eager.iterate()               # eager launches of the same library between the replays
        torch.cuda.synchronize()
        for i, (tr, te) in enumerate(zip(rec.outputs(), eager.outputs())):
            assert torch.equal(tr, te), (k, i)
        assert host(rec.ctr).tolist() == [(k + 1) * w.T, k + 1, (k + 1) * n, (k + 1) * n if w.rnd else 0]
    assert torch.isfinite(rec.actor.params).all()


class RecurrentLoop:
    """The recurrent training iteration (memories carried across iterations, reset at episode ends) on device
    counters, or on host counters for comparison."""

    def __init__(self, rx, w, inp, device_counters):
        self.rx, self.w, self.dc = rx, w, device_counters
        T, N, A, H = w.T, w.N, w.A, w.memory_hidden
        lstm = w.memory_cell == "lstm"
        cid, S = (rx.CELL_LSTM, 2 * H) if lstm else (rx.CELL_GRU, H)
        self.ga = rx.Memory(cid, w.Da, H, dev(inp["mem_actor"]), trainable=True)
        self.gc = rx.Memory(cid, w.Dc, H, dev(inp["mem_critic"]), trainable=True)
        self.ma = rx.Mlp(w.dims_actor, dev(inp["actor"]), trainable=True, has_log_std=True)
        self.mc = rx.Mlp(w.dims_critic, dev(inp["critic"]), trainable=True)
        self.obs, self.rewards, self.dones = dev(inp["obs"]), dev(inp["rewards"]), dev(inp["dones"])
        self.h_a, self.h_c = dev(inp["h_actor"]), dev(inp["h_critic"])
        self.h0_a, self.h0_c = torch.zeros(N, S, device="cuda"), torch.zeros(N, S, device="cuda")
        self.actions, self.mu, self.sigma = (torch.zeros(T, N, A, device="cuda") for _ in range(3))
        self.logp, self.values, self.adv, self.ret = (torch.zeros(T, N, device="cuda") for _ in range(4))
        self.last = torch.zeros(N, device="cuda")
        self.rollout = rx.Rollout(T, N, self.obs[:T], self.obs[:T], self.actions, self.logp, self.values, self.mu, self.sigma,
                                  self.adv, self.ret)
        self.cfg_kw = dict(clip=w.clip, value_coef=w.value_coef, entropy_coef=w.entropy_coef, max_grad_norm=w.max_grad_norm,
                           lr=w.lr, epochs=2, minibatches=w.minibatches, seed=SEED)
        self.stats = torch.zeros(2 * w.minibatches, rx.NSTATS, device="cuda")
        nets = (self.ga, self.ma, self.gc, self.mc)
        self.aws = rx.workspace(rx.rslx_act_recurrent_workspace_bytes(*nets, N))
        self.gws = rx.workspace(rx.rslx_gae_workspace_bytes(T, N))
        self.uws = rx.workspace(rx.rslx_ppo_update_recurrent_workspace_bytes(*nets, self.rollout, rx.PpoCfg(**self.cfg_kw)))
        self.act_step, self.call_index, self.adam_step = 0, 0, C.c_int64(0)
        self.ctr = rx.dev_counters() if device_counters else None
        self.state = [t.clone() for t in self.state_tensors()]

    def state_tensors(self):
        ts = [self.h_a, self.h_c]
        for n in (self.ga, self.ma, self.gc, self.mc):
            ts += [n.params, n.adam_m, n.adam_v]
        if self.ctr is not None:
            ts.append(self.ctr)
        return ts

    def reset(self):
        for t, t0 in zip(self.state_tensors(), self.state):
            t.copy_(t0)

    def outputs(self):
        return [self.actions, self.mu, self.sigma, self.logp, self.values, self.last, self.adv, self.ret, self.stats, self.h0_a,
                self.h0_c, self.h_a, self.h_c, self.ga.params, self.ma.params, self.gc.params, self.mc.params, self.ga.adam_v]

    def iterate(self):
        rx, w = self.rx, self.w
        T, N = w.T, w.N
        nets = (self.ga, self.ma, self.gc, self.mc)
        for t in range(T):
            o = self.obs[t]
            reset = self.dones[t - 1] if t > 0 else self.dones[T - 1]       # the previous roll-out ended with these flags
            h0 = (self.h0_a, self.h0_c) if t == 0 else (None, None)
            outs = (self.actions[t], self.logp[t], self.values[t], self.mu[t], self.sigma[t])
            if self.dc:
                rx.rslx_act_recurrent_dc(*nets, o, o, N, self.h_a, self.h_c, reset, *h0, SEED, self.ctr, None, *outs, 0, self.aws)
            else:
                rx.rslx_act_recurrent(*nets, o, o, N, self.h_a, self.h_c, reset, *h0, SEED, self.act_step, None, *outs, 0, self.aws)
                self.act_step += 1
        rx.rslx_act_recurrent(None, None, self.gc, self.mc, None, self.obs[T], N, None, self.h_c, self.dones[T - 1], None, None, 0, 0,
                              None, None, None, self.last, None, None, rx.ACT_VALUES_ONLY, self.aws)
        rx.rslx_gae(self.rewards, self.values, self.last, self.dones, None, T, N, w.gamma, w.lam, 1, self.adv, self.ret, self.gws)
        if self.dc:
            rx.rslx_ppo_update_recurrent_dc(*nets, self.rollout, self.dones, self.h0_a, self.h0_c, rx.PpoCfg(**self.cfg_kw), self.ctr,
                                            self.stats, self.uws)
        else:
            rx.rslx_ppo_update_recurrent(*nets, self.rollout, self.dones, self.h0_a, self.h0_c,
                                         rx.PpoCfg(call_index=self.call_index, **self.cfg_kw), self.adam_step, self.stats, self.uws)
            self.call_index += 1


@pytest.mark.parametrize("cell", ["gru", "lstm"])
def test_recurrent_iteration_on_device_counters_and_as_a_graph(rx, cell):
    w = replace(WORKLOADS["recurrent"].scaled(64), hidden=(64, 32), memory_hidden=32, done_p=0.05, memory_cell=cell)
    inp = make_inputs(w)
    n = 2 * w.minibatches
    # device counters against host counters (Adam's bias corrections differ in the last bit at most)
    h, d = RecurrentLoop(rx, w, inp, False), RecurrentLoop(rx, w, inp, True)
    for it in range(2):
        h.iterate(); d.iterate()
        torch.cuda.synchronize()
        if it == 0:
            assert torch.equal(h.actions, d.actions) and torch.equal(h.h0_a, d.h0_a)
        for th, td in zip(h.outputs(), d.outputs()):
            assert rel_l2(host(td), host(th)) <= 1e-5
        assert host(d.ctr).tolist() == [(it + 1) * w.T, it + 1, (it + 1) * n, 0]
    # graph replays against the eager device-counter loop, bit for bit
    eager, rec = RecurrentLoop(rx, w, inp, True), RecurrentLoop(rx, w, inp, True)
    rec.iterate()
    torch.cuda.synchronize()
    rec.reset()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rec.iterate()
    torch.cuda.synchronize()
    assert host(rec.ctr).tolist() == [0, 0, 0, 0]
    for k in range(3):
        g.replay()
        eager.iterate()
        torch.cuda.synchronize()
        for i, (tr, te) in enumerate(zip(rec.outputs(), eager.outputs())):
            assert torch.equal(tr, te), (k, i)
        assert host(rec.ctr).tolist() == [(k + 1) * w.T, k + 1, (k + 1) * n, 0]
