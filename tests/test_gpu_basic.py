"""GPU parity: permutation (bit-exact), GAE, Adam, act(), symmetry augmentation, RND reward vs the fp64 oracle."""
import ctypes as C
import numpy as np
import pytest
import torch

from oracle import rng as orng, gae as ogae, adam as oadam, ppo as oppo, symmetry as osym, rnd as ornd, mlp as omlp
from workloads import WORKLOADS, make_inputs, random_involution
from gpu_util import dev, host, rel_l2, f32, assert_elementwise

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rx():
    import paper_2509_10771_amd as m
    m.rslx_device_check()
    return m


@pytest.mark.parametrize("B", [1, 2, 63, 64, 65, 1536, 4097, 98304, 393216])
def test_permutation_bit_exact(rx, B):
    ws = rx.workspace(rx.rslx_permutation_workspace_bytes(B))
    out = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    for (seed, call, epoch) in [(20250910, 1, 0), (0, 0, 4)]:
        rx.rslx_permutation(seed, call, epoch, B, out, ws)
        torch.cuda.synchronize()
        assert np.array_equal(host(out), orng.permutation(seed, call, epoch, B))


def _gae_case(rx, T, N, gamma, lam, p_done, timeouts, normalize, seed=0):
    g = np.random.default_rng(seed)
    r = g.normal(0.5, 0.3, size=(T, N)).astype(np.float32); V = g.normal(size=(T, N)).astype(np.float32)
    Vl = g.normal(size=N).astype(np.float32); d = (g.random((T, N)) < p_done).astype(np.uint8)
    to = (d * (g.random((T, N)) < 0.5)).astype(np.uint8) if timeouts else None
    adv = torch.empty(T, N, device="cuda"); ret = torch.empty(T, N, device="cuda")
    ws = rx.workspace(rx.rslx_gae_workspace_bytes(T, N))
    rx.rslx_gae(dev(r), dev(V), dev(Vl), dev(d), dev(to) if timeouts else None, T, N, gamma, lam, normalize, adv, ret, ws)
    torch.cuda.synchronize()
    a_ref, r_ref = ogae.gae(r, V, Vl, d, gamma, lam, timeouts=to)
    assert np.max(np.abs(host(ret) - r_ref) / np.maximum(np.abs(r_ref), 1.0)) <= 1e-5
    if normalize:
        z_ref = ogae.normalize_advantages(a_ref)
        assert np.max(np.abs(host(adv) - z_ref)) <= 2e-5 * max(1.0, np.abs(z_ref).max())
    else:
        assert np.max(np.abs(host(adv) - a_ref) / np.maximum(np.abs(a_ref), 1.0)) <= 1e-5


@pytest.mark.parametrize("T,N", [(1, 1), (24, 64), (24, 100), (7, 4096), (24, 16384), (24, 70001)])
def test_gae_matches_oracle(rx, T, N):
    _gae_case(rx, T, N, 0.99, 0.95, 0.02, False, False)
    _gae_case(rx, T, N, 0.99, 0.95, 0.3, True, T * N > 1, seed=1)


def test_gae_edge_cases(rx):
    _gae_case(rx, 24, 333, 0.0, 0.95, 0.1, False, False)
    _gae_case(rx, 24, 333, 0.99, 1.0, 0.0, False, True)
    _gae_case(rx, 24, 333, 0.99, 0.95, 1.0, True, True)
    rx.rslx_gae(None, None, None, None, None, 0, 5, 0.9, 0.9, 1, None, None, None)     # empty rollout


@pytest.mark.parametrize("n", [1, 5, 1023, 1024, 380313, 1 << 20])
def test_adam_matches_oracle(rx, n):
    g = np.random.default_rng(n)
    th = g.normal(size=n).astype(np.float32); gr = (g.normal(size=n) * 0.01).astype(np.float32)
    pad = lambda x: dev(x)
    for max_norm in (1.0, 0.0):
        p, gg, m, v = pad(th), pad(gr), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
        step = C.c_int64(0)
        norm_out = torch.zeros(1, device="cuda")
        ws = rx.workspace(rx.rslx_adam_workspace_bytes(n))
        ref = (th.astype(np.float64), np.zeros(n), np.zeros(n), 0)
        for k in range(3):
            rx.rslx_adam_step(p, gg, m, v, n, 1e-3, 0.9, 0.999, 1e-8, max_norm, step, norm_out, ws)
            norm = oadam.global_norm([gr])
            s = oadam.clip_scale(norm, max_norm)
            ref = oadam.adam_step(ref[0], s * gr.astype(np.float64), ref[1], ref[2], ref[3], f32(1e-3), f32(0.9), f32(0.999), f32(1e-8))
        torch.cuda.synchronize()
        assert step.value == 3
        assert abs(host(norm_out)[0] - norm) <= 1e-5 * norm
        np.testing.assert_allclose(host(p), ref[0], rtol=2e-6, atol=2e-7)
        np.testing.assert_allclose(host(m), ref[1], rtol=1e-5, atol=1e-10)
        np.testing.assert_allclose(host(v), ref[2], rtol=1e-5, atol=1e-14)


def _act_case(rx, w, inp, N, use_eps, step=5, seed=11):
    actor = rx.Mlp(w.dims_actor, dev(inp["actor"]), has_log_std=True)
    critic = rx.Mlp(w.dims_critic, dev(inp["critic"]))
    obs = inp["obs"][0][:N]
    A = w.A
    eps = orng.act_noise(seed, step, N, A)
    out = {k: torch.empty(N, A, device="cuda") for k in ("actions", "mu", "sigma")}
    logp = torch.empty(N, device="cuda"); values = torch.empty(N, device="cuda")
    ws = rx.workspace(rx.rslx_act_workspace_bytes(actor, critic, N))
    d_obs = dev(obs)
    rx.rslx_act(actor, critic, d_obs, d_obs, N, seed, step, dev(eps.astype(np.float32)) if use_eps else None,
                out["actions"], logp, values, out["mu"], out["sigma"], 0, ws)
    torch.cuda.synchronize()
    ref = oppo.act(inp["actor"], inp["critic"], w.dims_actor, w.dims_critic, obs, obs,
                   eps.astype(np.float32) if use_eps else eps)
    scale = max(1.0, np.abs(ref["mu"]).max())
    assert np.abs(host(out["mu"]) - ref["mu"]).max() <= 2e-5 * scale
    assert np.abs(host(values) - ref["values"]).max() <= 2e-5 * max(1.0, np.abs(ref["values"]).max())
    assert np.abs(host(out["sigma"]) - ref["sigma"]).max() <= 1e-6
    assert np.abs(host(out["actions"]) - ref["actions"]).max() <= 3e-5 * scale
    assert np.abs(host(logp) - ref["logp"]).max() <= 1e-4 * max(1.0, np.abs(ref["logp"]).max())
    # values-only and deterministic flags
    v2 = torch.empty(N, device="cuda")
    rx.rslx_act(None, critic, None, d_obs, N, 0, 0, None, None, None, v2, None, None, rx.ACT_VALUES_ONLY, ws)
    a2 = torch.empty(N, A, device="cuda")
    rx.rslx_act(actor, critic, d_obs, d_obs, N, 0, 0, None, a2, logp, values, out["mu"], out["sigma"], rx.ACT_DETERMINISTIC, ws)
    torch.cuda.synchronize()
    assert torch.equal(v2, values) and torch.equal(a2, out["mu"])


@pytest.mark.parametrize("name,N", [("tiny", 64), ("flat", 300), ("flat", 4096), ("rough", 257), ("rough", 4096)])
def test_act_matches_oracle(rx, name, N):
    w = WORKLOADS[name].scaled(max(N, 1))
    inp = make_inputs(w)
    inp["actor"][-w.A:] = np.random.default_rng(0).normal(scale=0.3, size=w.A).astype(np.float32)   # non-trivial log_std
    _act_case(rx, w, inp, N, use_eps=True)
    _act_case(rx, w, inp, N, use_eps=False)


@pytest.mark.parametrize("name,N", [("flat", 8192), ("flat", 8193), ("curiosity", 16384)])
def test_act_large_batches_switch_to_the_per_layer_launches(rx, name, N):
    """Up to 8192 rows (256 row blocks per network) the layer-fused launch is used, beyond that the tiled per-layer
    launches: the same outputs either side of the switch and at the curiosity workload's size."""
    w = WORKLOADS[name].scaled(N)
    inp = make_inputs(w)
    inp["actor"][-w.A:] = np.random.default_rng(2).normal(scale=0.3, size=w.A).astype(np.float32)
    _act_case(rx, w, inp, N, use_eps=False)


def test_act_wide_layers_take_the_layered_path(rx):
    """Hidden layers wider than 512 do not fit the layer-fused kernel's LDS budget; the per-layer path must agree too."""
    from dataclasses import replace
    w = replace(WORKLOADS["tiny"], N=200, hidden=(640, 96))
    inp = make_inputs(w)
    _act_case(rx, w, inp, 200, use_eps=True)
    _act_case(rx, w, inp, 200, use_eps=False)


@pytest.mark.parametrize("Da,hidden,A", [(45, (100, 36), 7), (3, (8,), 1), (130, (192, 320, 20), 5), (48, (512, 512), 33)])
def test_act_odd_shapes_in_the_fused_kernel(rx, Da, hidden, A):
    """Widths that are no multiple of 4 or 64: ragged contraction tails, unaligned rows (scalar weight loads),
    column groups that end inside a 64-column task, contraction ranges that split unevenly over wavefronts."""
    from dataclasses import replace
    w = replace(WORKLOADS["tiny"], N=77, Da=Da, Dc=Da, A=A, hidden=hidden)
    inp = make_inputs(w)
    inp["actor"][-w.A:] = np.random.default_rng(1).normal(scale=0.3, size=w.A).astype(np.float32)
    _act_case(rx, w, inp, 77, use_eps=True)
    _act_case(rx, w, inp, 77, use_eps=False)


def test_act_noise_distribution(rx):
    w = WORKLOADS["flat"]
    inp = make_inputs(w)
    actor = rx.Mlp(w.dims_actor, dev(inp["actor"]), has_log_std=True); critic = rx.Mlp(w.dims_critic, dev(inp["critic"]))
    N, A = w.N, w.A
    d_obs = dev(inp["obs"][0])
    acts, mu, sg = (torch.empty(N, A, device="cuda") for _ in range(3))
    logp, values = torch.empty(N, device="cuda"), torch.empty(N, device="cuda")
    ws = rx.workspace(rx.rslx_act_workspace_bytes(actor, critic, N))
    rx.rslx_act(actor, critic, d_obs, d_obs, N, 123, 9, None, acts, logp, values, mu, sg, 0, ws)
    torch.cuda.synchronize()
    eps = host((acts - mu) / sg)
    np.testing.assert_allclose(eps, orng.act_noise(123, 9, N, A), atol=2e-5)
    assert abs(eps.mean()) < 2e-2 and abs(eps.var() - 1) < 2e-2


@pytest.mark.parametrize("B,D,A", [(1, 5, 3), (1000, 48, 12), (4099, 235, 12)])
def test_sym_augment(rx, B, D, A):
    g = np.random.default_rng(B)
    po, so = random_involution(g, D); pa, sa = random_involution(g, A)
    sym = rx.Sym(po, so, po, so, pa, sa)
    obs = g.normal(size=(B, D)).astype(np.float32); act = g.normal(size=(B, A)).astype(np.float32)
    o2 = torch.empty(2 * B, D, device="cuda"); a2 = torch.empty(2 * B, A, device="cuda")
    rx.rslx_sym_augment(sym, dev(obs), dev(act), B, D, A, o2, a2)
    torch.cuda.synchronize()
    ro, ra = osym.augment(obs, act, po, so, pa, sa)
    assert np.array_equal(host(o2), ro.astype(np.float32)) and np.array_equal(host(a2), ra.astype(np.float32))


@pytest.mark.parametrize("N,subset", [(64, False), (1000, True), (16384, False)])
def test_rnd_reward(rx, N, subset):
    w = WORKLOADS["curiosity"].scaled(N)
    inp = make_inputs(w)
    D = w.Da
    g = np.random.default_rng(1)
    dims = w.dims_rnd
    sub = None
    if subset:
        sub = np.sort(g.choice(D, size=20, replace=False)).astype(np.int32)
        dims = (20,) + dims[1:]
        from workloads import xavier_mlp
        inp["rnd_target"], inp["rnd_predictor"] = xavier_mlp(g, dims), xavier_mlp(g, dims)
    targ = rx.Mlp(dims, dev(inp["rnd_target"])); pred = rx.Mlp(dims, dev(inp["rnd_predictor"]))
    running = dev(np.array([0.0, 1.0, 1e-4], np.float32))
    ws = rx.workspace(rx.rslx_rnd_workspace_bytes(targ, N))
    run_ref = (0.0, 1.0, 1e-4)
    for t in range(3):
        obs = inp["obs"][t]
        rew = inp["rewards"][t].copy()
        d_rew = dev(rew); r_int = torch.empty(N, device="cuda")
        rx.rslx_rnd(targ, pred, dev(obs), N, D, dev(sub) if subset else None, dims[0], running, 0.5, 1, r_int, d_rew, ws)
        torch.cuda.synchronize()
        ri_ref, raw_ref, run_ref = ornd.intrinsic_reward(inp["rnd_predictor"], inp["rnd_target"], dims, obs, run_ref, sub)
        assert rel_l2(host(r_int), ri_ref) < 1e-4
        assert_elementwise("r_int[%d]" % t, host(r_int), ri_ref)
        np.testing.assert_allclose(host(d_rew), rew + 0.5 * ri_ref, rtol=1e-4, atol=1e-5)
        np.testing.assert_allclose(host(running), np.array(run_ref), rtol=1e-4)
    # frozen statistics
    before = host(running).copy()
    rx.rslx_rnd(targ, pred, dev(inp["obs"][3]), N, D, dev(sub) if subset else None, dims[0], running, 0.5, 0, r_int, None, ws)
    torch.cuda.synchronize()
    assert np.array_equal(host(running), before)
    ri_ref, _, _ = ornd.intrinsic_reward(inp["rnd_predictor"], inp["rnd_target"], dims, inp["obs"][3], run_ref, sub, update_stats=False)
    assert rel_l2(host(r_int), ri_ref) < 1e-4
    assert_elementwise("r_int (frozen statistics)", host(r_int), ri_ref)
