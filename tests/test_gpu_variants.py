"""GPU parity on the two workload variants that reach paths the five main configurations leave cold:
episodes cut by a time limit next to early terminations (paper Sec. 3, timeouts are bootstrapped, terminations are
not) and RND on a strict subset of the state (paper Sec. 2.2).

The collection loop (act, intrinsic reward, value bootstrap, advantage estimation) runs on the GPU with the oracle's
noise handed in, and every buffer it fills is compared with the oracle's; the update is then checked by the same
step-forced and free-running comparisons as the main workloads.
"""
import numpy as np
import pytest
import torch

from oracle import ppo as oppo, gae as ogae, rng as orng, rnd as ornd
from workloads import WORKLOADS, make_inputs
from gpu_util import dev, host, rel_l2
from test_gpu_update import Case, check_forced_steps, check_free_running

pytestmark = pytest.mark.gpu

SEED = 9


@pytest.fixture(scope="module")
def rx():
    import paper_2509_10771_amd as m
    m.rslx_device_check()
    return m


def oracle_collect(w, inp):
    T, N, A = w.T, w.N, w.A
    sub = inp.get("rnd_subset_idx")
    rewards = np.asarray(inp["rewards"], np.float64).copy()
    running = (0.0, 1.0, 1e-4)
    out = dict(actions=[], logp=[], values=[], r_int=[])
    for t in range(T):
        o = oppo.act(inp["actor"], inp["critic"], w.dims_actor, w.dims_critic, inp["obs"][t], inp["obs"][t],
                     orng.act_noise(SEED, t, N, A))
        for k in ("actions", "logp", "values"):
            out[k].append(o[k])
        if w.rnd:
            ri, _, running = ornd.intrinsic_reward(inp["rnd_predictor"], inp["rnd_target"], w.dims_rnd, inp["obs"][t],
                                                   running, sub)
            rewards[t] += w.rnd_weight * ri
            out["r_int"].append(ri)
    last = oppo.act(inp["actor"], inp["critic"], w.dims_actor, w.dims_critic, inp["obs"][T], inp["obs"][T],
                    np.zeros((N, A)))["values"]
    values = np.stack(out["values"])
    adv, ret = ogae.gae(rewards, values, last, inp["dones"], w.gamma, w.lam, timeouts=inp.get("timeouts"))
    return dict(actions=np.stack(out["actions"]), logp=np.stack(out["logp"]), values=values, last=last, rewards=rewards,
                adv_raw=adv, adv=ogae.normalize_advantages(adv), ret=ret, running=running)


def gpu_collect(rx, w, inp, normalize):
    T, N, A = w.T, w.N, w.A
    actor = rx.Mlp(w.dims_actor, dev(inp["actor"]), has_log_std=True)
    critic = rx.Mlp(w.dims_critic, dev(inp["critic"]))
    obs, rewards, dones = dev(inp["obs"]), dev(inp["rewards"]), dev(inp["dones"])
    timeouts = dev(inp["timeouts"]) if "timeouts" in inp else None
    sub = dev(inp["rnd_subset_idx"]) if "rnd_subset_idx" in inp else None
    actions, mu, sigma = (torch.empty(T, N, A, device="cuda") for _ in range(3))
    logp, values, adv, ret = (torch.empty(T, N, device="cuda") for _ in range(4))
    last = torch.empty(N, device="cuda")
    aws = rx.workspace(rx.rslx_act_workspace_bytes(actor, critic, N))
    gws = rx.workspace(rx.rslx_gae_workspace_bytes(T, N))
    if w.rnd:
        rt, rp = rx.Mlp(w.dims_rnd, dev(inp["rnd_target"])), rx.Mlp(w.dims_rnd, dev(inp["rnd_predictor"]))
        running = dev(np.array([0.0, 1.0, 1e-4], np.float32))
        r_int = torch.empty(N, device="cuda")
        rws = rx.workspace(rx.rslx_rnd_workspace_bytes(rt, N))
    for t in range(T):
        eps = dev(orng.act_noise(SEED, t, N, A), torch.float32)
        rx.rslx_act(actor, critic, obs[t], obs[t], N, SEED, t, eps, actions[t], logp[t], values[t], mu[t], sigma[t], 0, aws)
        if w.rnd:
            rx.rslx_rnd(rt, rp, obs[t], N, w.Da, sub, w.dims_rnd[0], running, w.rnd_weight, 1, r_int, rewards[t], rws)
    rx.rslx_act(None, critic, None, obs[T], N, 0, 0, None, None, None, last, None, None, rx.ACT_VALUES_ONLY, aws)
    rx.rslx_gae(rewards, values, last, dones, timeouts, T, N, w.gamma, w.lam, int(normalize), adv, ret, gws)
    torch.cuda.synchronize()
    return dict(actions=host(actions), logp=host(logp), values=host(values), last=host(last), rewards=host(rewards),
                adv=host(adv), ret=host(ret), running=host(running) if w.rnd else None)


@pytest.mark.parametrize("name,N", [("flat_timeouts", 300), ("curiosity_subset", 200), ("flat_timeouts", 4096)])
def test_collection_loop_matches_oracle(rx, name, N):
    w = WORKLOADS[name].scaled(N)
    inp = make_inputs(w)
    if "timeouts" in inp:      # both kinds of episode end are present
        assert inp["timeouts"].sum() > 0 and (inp["dones"] & ~inp["timeouts"]).sum() > 0
    ref = oracle_collect(w, inp)
    for normalize in (False, True):
        got = gpu_collect(rx, w, inp, normalize)
        for k in ("actions", "logp", "values", "last"):
            assert rel_l2(got[k], ref[k]) <= 1e-5, k
        if w.rnd:
            assert rel_l2(got["rewards"], ref["rewards"]) <= 1e-4
            np.testing.assert_allclose(got["running"], np.array(ref["running"]), rtol=1e-4)
        # the scan itself is checked to 1e-5 on identical inputs elsewhere; here its inputs carry the forward pass's
        # fp32 rounding (and, with RND, the intrinsic reward's 1e-4), which the bound below allows for
        tol = 1e-4 if w.rnd else 2e-5
        assert np.max(np.abs(got["ret"] - ref["ret"])) <= tol * max(1.0, np.max(np.abs(ref["ret"])))
        want = ref["adv"] if normalize else ref["adv_raw"]
        assert np.max(np.abs(got["adv"] - want)) <= tol * max(1.0, np.max(np.abs(want)))


def test_ppo_update_after_timeouts(rx):
    case = Case(WORKLOADS["flat_timeouts"].scaled(250), 1)
    check_free_running(rx, case, check_forced_steps(rx, case))


def test_ppo_update_with_workload_rnd_subset(rx):
    from dataclasses import replace
    case = Case(replace(WORKLOADS["curiosity_subset"].scaled(168), minibatches=4), 1, rnd_on=True)
    assert case.rnd_sub is not None and len(case.rnd_sub) == 24
    check_free_running(rx, case, check_forced_steps(rx, case))
