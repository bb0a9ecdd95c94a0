"""End-to-end check that the whole loop (act, reward, GAE, update) actually optimises something: a synthetic
one-step control task whose reward is minus the squared distance between the action and a fixed linear function of
the observation.  No oracle here (parity is the business of the other test files); what is checked is the
direction: after a few dozen iterations the mean reward is much higher than at the start, for the feed-forward
networks, for both recurrent memories, and for the distillation of the trained policy's target into a student."""
import ctypes as C
import numpy as np
import pytest
import torch

from workloads import xavier_mlp, uniform_memory

pytestmark = pytest.mark.gpu

N, T, D, A, HID = 256, 8, 6, 2, (32, 32)


@pytest.fixture(scope="module")
def rx():
    import paper_2509_10771_amd as m
    m.rslx_device_check()
    return m


def _task(seed=0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    target_map = (0.7 * torch.randn(D, A, generator=g)).cuda()

    def sample_obs(it):
        gg = torch.Generator(device="cpu").manual_seed(1000 + it)
        return torch.randn(T + 1, N, D, generator=gg).cuda()

    def reward(obs, actions):
        return -((actions - obs @ target_map) ** 2).sum(-1)

    return sample_obs, reward, target_map


def _cfg(rx, it):
    return rx.PpoCfg(clip=0.2, value_coef=1.0, entropy_coef=0.0, max_grad_norm=1.0, lr=3e-3, epochs=4, minibatches=4, seed=5,
                     call_index=it)


def test_feed_forward_ppo_improves_the_reward(rx):
    g = np.random.default_rng(0)
    dims_a, dims_c = (D,) + HID + (A,), (D,) + HID + (1,)
    actor = rx.Mlp(dims_a, torch.from_numpy(xavier_mlp(g, dims_a, log_std=True)).cuda(), trainable=True, has_log_std=True)
    critic = rx.Mlp(dims_c, torch.from_numpy(xavier_mlp(g, dims_c)).cuda(), trainable=True)
    sample_obs, reward, _ = _task()
    actions, mu, sigma = (torch.empty(T, N, A, device="cuda") for _ in range(3))
    logp, values, adv, ret = (torch.empty(T, N, device="cuda") for _ in range(4))
    last = torch.empty(N, device="cuda")
    dones = torch.ones(T, N, dtype=torch.uint8, device="cuda")          # one-step episodes
    stats = torch.zeros(16, rx.NSTATS, device="cuda")
    aws = rx.workspace(rx.rslx_act_workspace_bytes(actor, critic, N))
    gws = rx.workspace(rx.rslx_gae_workspace_bytes(T, N))
    step = C.c_int64(0)
    history = []
    for it in range(40):
        obs = sample_obs(it)
        for t in range(T):
            rx.rslx_act(actor, critic, obs[t], obs[t], N, 11, it * T + t, None, actions[t], logp[t], values[t], mu[t], sigma[t], 0, aws)
        rx.rslx_act(None, critic, None, obs[T], N, 0, 0, None, None, None, last, None, None, rx.ACT_VALUES_ONLY, aws)
        rew = reward(obs[:T], actions).contiguous()
        history.append(float(rew.mean()))
        rx.rslx_gae(rew, values, last, dones, None, T, N, 0.99, 0.95, 1, adv, ret, gws)
        ro = rx.Rollout(T, N, obs[:T], obs[:T], actions, logp, values, mu, sigma, adv, ret)
        cfg = _cfg(rx, it)
        uws = rx.workspace(rx.rslx_ppo_update_workspace_bytes(actor, critic, ro, cfg))
        rx.rslx_ppo_update(actor, critic, ro, cfg, None, None, step, stats, uws)
    torch.cuda.synchronize()
    print("mean reward per iteration:", [round(h, 2) for h in history[::5]])
    assert step.value == 40 * 16 and torch.isfinite(actor.params).all()
    assert np.mean(history[-5:]) > 0.1 * np.mean(history[:3])         # rewards are negative: less than 10 % of the first loss is left
    # (measured: -8.1 at the start, -0.08 after 40 iterations)


@pytest.mark.parametrize("cell", ["gru", "lstm"])
def test_recurrent_ppo_improves_a_reward_that_needs_memory(rx, cell):
    """The rewarded action depends on the PREVIOUS step's observation, which only the memory can supply."""
    g = np.random.default_rng(1)
    H = 32
    G, S = (4, 2 * H) if cell == "lstm" else (3, H)
    cid = rx.CELL_LSTM if cell == "lstm" else rx.CELL_GRU
    dims_a, dims_c = (H,) + HID + (A,), (H,) + HID + (1,)
    ga = rx.Memory(cid, D, H, torch.from_numpy(uniform_memory(g, D, H, G)).cuda(), trainable=True)
    gc = rx.Memory(cid, D, H, torch.from_numpy(uniform_memory(g, D, H, G)).cuda(), trainable=True)
    ma = rx.Mlp(dims_a, torch.from_numpy(xavier_mlp(g, dims_a, log_std=True)).cuda(), trainable=True, has_log_std=True)
    mc = rx.Mlp(dims_c, torch.from_numpy(xavier_mlp(g, dims_c)).cuda(), trainable=True)
    sample_obs, _, target_map = _task(3)
    actions, mu, sigma = (torch.empty(T, N, A, device="cuda") for _ in range(3))
    logp, values, adv, ret = (torch.empty(T, N, device="cuda") for _ in range(4))
    last = torch.empty(N, device="cuda")
    dones = torch.zeros(T, N, dtype=torch.uint8, device="cuda")
    h_a, h_c = torch.zeros(N, S, device="cuda"), torch.zeros(N, S, device="cuda")
    h0_a, h0_c = torch.zeros(N, S, device="cuda"), torch.zeros(N, S, device="cuda")
    reset_all = torch.ones(N, dtype=torch.uint8, device="cuda")        # every roll-out is a fresh episode
    stats = torch.zeros(8, rx.NSTATS, device="cuda")
    aws = rx.workspace(rx.rslx_act_recurrent_workspace_bytes(ga, ma, gc, mc, N))
    gws = rx.workspace(rx.rslx_gae_workspace_bytes(T, N))
    step = C.c_int64(0)
    history = []
    for it in range(60):
        obs = sample_obs(it)
        for t in range(T):
            rx.rslx_act_recurrent(ga, ma, gc, mc, obs[t], obs[t], N, h_a, h_c, reset_all if t == 0 else None,
                                  h0_a if t == 0 else None, h0_c if t == 0 else None, 11, it * T + t, None, actions[t], logp[t],
                                  values[t], mu[t], sigma[t], 0, aws)
        rx.rslx_act_recurrent(None, None, gc, mc, None, obs[T], N, None, h_c, None, None, None, 0, 0, None, None, None, last, None,
                              None, rx.ACT_VALUES_ONLY, aws)
        prev = torch.cat([torch.zeros(1, N, D, device="cuda"), obs[:T - 1]])
        rew = (-((actions - prev @ target_map) ** 2).sum(-1)).contiguous()
        history.append(float(rew[1:].mean()))
        rx.rslx_gae(rew, values, last, dones, None, T, N, 0.0, 0.95, 1, adv, ret, gws)      # gamma = 0: each step is its own problem
        ro = rx.Rollout(T, N, obs[:T], obs[:T], actions, logp, values, mu, sigma, adv, ret)
        cfg = rx.PpoCfg(clip=0.2, value_coef=1.0, entropy_coef=0.0, max_grad_norm=1.0, lr=3e-3, epochs=4, minibatches=2, seed=5,
                        call_index=it)
        uws = rx.workspace(rx.rslx_ppo_update_recurrent_workspace_bytes(ga, ma, gc, mc, ro, cfg))
        rx.rslx_ppo_update_recurrent(ga, ma, gc, mc, ro, dones, h0_a, h0_c, cfg, step, stats, uws)
    torch.cuda.synchronize()
    print("mean reward per iteration:", [round(h, 2) for h in history[::6]])
    assert torch.isfinite(ga.params).all() and torch.isfinite(ma.params).all()
    assert np.mean(history[-5:]) > 0.15 * np.mean(history[:3])        # measured: -6.4 at the start, -0.2 after 60 iterations


def test_distillation_brings_the_student_to_the_teacher(rx):
    g = np.random.default_rng(2)
    dims_t, dims_s = (D,) + HID + (A,), (D, 16, A)
    teacher = rx.Mlp(dims_t, torch.from_numpy(xavier_mlp(g, dims_t)).cuda())
    student = rx.Mlp(dims_s, torch.from_numpy(xavier_mlp(g, dims_s)).cuda(), trainable=True)
    sample_obs, _, _ = _task(4)
    actions, targets = torch.empty(T, N, A, device="cuda"), torch.empty(T, N, A, device="cuda")
    cfg_kw = dict(lr=3e-3, epochs=2, minibatches=4, seed=3)
    stats = torch.zeros(8, rx.NSTATS, device="cuda")
    cws = rx.workspace(rx.rslx_bc_collect_workspace_bytes(student, teacher, N))
    uws = rx.workspace(rx.rslx_bc_update_workspace_bytes(student, None, T * N, rx.BcCfg(**cfg_kw)))
    step = C.c_int64(0)
    losses = []
    for it in range(40):
        obs = sample_obs(it)[:T].contiguous()
        for t in range(T):
            rx.rslx_bc_collect(student, teacher, obs[t], obs[t], N, actions[t], targets[t], cws)
        losses.append(float(((actions - targets) ** 2).mean()))
        rx.rslx_bc_update(student, None, obs, None, targets, T * N, rx.BcCfg(call_index=it, **cfg_kw), step, stats, uws)
    torch.cuda.synchronize()
    print("student-teacher mse per iteration:", [round(l, 4) for l in losses[::5]])
    assert losses[-1] < 0.1 * losses[0]
