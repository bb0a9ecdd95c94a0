"""Shared helpers of the GPU parity tests: oracle-built rollouts and device marshalling."""
import ctypes
import numpy as np
import torch

from oracle import ppo as oppo, gae as ogae, rng as orng
from workloads import make_inputs


def dev(x, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda().contiguous()


def host(t):
    return t.detach().cpu().numpy()


def rel_l2(x, ref):
    x, ref = np.asarray(x, np.float64).ravel(), np.asarray(ref, np.float64).ravel()
    return float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-30))


def assert_elementwise(name, got, ref, rtol=1e-4, atol_frac=1e-5):
    """|got - ref| <= rtol |ref| + atol_frac max|ref| for every element (the absolute part covers entries that are
    sums of cancelling terms, whose fp32 error is relative to the terms)."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    if ref.size == 0:
        return
    err = np.abs(got - ref)
    bound = rtol * np.abs(ref) + atol_frac * np.abs(ref).max() + 1e-30
    if np.any(err > bound):
        i = np.unravel_index(int(np.argmax(err / bound)), err.shape)
        raise AssertionError("%s%s: got %.9g ref %.9g (err %.3g, bound %.3g; %d of %d elements out)" % (
            name, list(i), got[i], ref[i], err[i], bound[i], int((err > bound).sum()), err.size))


def oracle_rollout(w, inp, seed=7, normalize=True):
    """Roll the oracle's act() over the T observation slabs; GAE by the oracle.  All outputs float32
    (what both implementations are then fed), flattened to B = T*N rows."""
    T, N, A = w.T, w.N, w.A
    obs = inp["obs"]
    acts, logp, vals, mu, sg = [], [], [], [], []
    for t in range(T):
        o = oppo.act(inp["actor"], inp["critic"], w.dims_actor, w.dims_critic, obs[t], obs[t], orng.act_noise(seed, t, N, A))
        acts.append(o["actions"]); logp.append(o["logp"]); vals.append(o["values"]); mu.append(o["mu"]); sg.append(o["sigma"])
    last = oppo.act(inp["actor"], inp["critic"], w.dims_actor, w.dims_critic, obs[T], obs[T], np.zeros((N, A)))["values"]
    f32 = lambda x: np.ascontiguousarray(np.asarray(x, np.float32))
    ro = dict(actions=f32(np.stack(acts)), logp=f32(np.stack(logp)), values=f32(np.stack(vals)), mu=f32(np.stack(mu)),
              sigma=f32(np.stack(sg)), last_values=f32(last))
    adv, ret = ogae.gae(inp["rewards"], ro["values"], ro["last_values"], inp["dones"], w.gamma, w.lam,
                        timeouts=inp.get("timeouts"))
    ro["adv_raw"], ro["returns"] = f32(adv), f32(ret)
    ro["adv"] = f32(ogae.normalize_advantages(adv)) if normalize else f32(adv)
    return ro


def flat_rollout(w, inp, ro):
    """Dict of [B, ...] float32 arrays in the oracle's update format."""
    B = w.B
    return dict(obs_a=inp["obs"][:w.T].reshape(B, -1), obs_c=inp["obs"][:w.T].reshape(B, -1),
                actions=ro["actions"].reshape(B, -1), logp=ro["logp"].reshape(B), values=ro["values"].reshape(B),
                mu=ro["mu"].reshape(B, -1), sigma=ro["sigma"].reshape(B, -1), adv=ro["adv"].reshape(B),
                returns=ro["returns"].reshape(B))


def f32(x):
    """A hyper-parameter as the fp32 value the C ABI carries (the oracle is fed the same number)."""
    return float(np.float32(x))


def oracle_cfg(w, epochs, seed=3, call_index=1):
    return oppo.PPOConfig(clip=f32(w.clip), value_coef=f32(w.value_coef), entropy_coef=f32(w.entropy_coef),
                          max_grad_norm=f32(w.max_grad_norm), lr=f32(w.lr), beta1=f32(0.9), beta2=f32(0.999),
                          adam_eps=f32(1e-8), epochs=epochs, minibatches=w.minibatches, seed=seed, call_index=call_index)
