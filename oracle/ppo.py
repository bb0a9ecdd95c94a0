"""PPO: act(), the minibatch loss with its gradient, and the multi-epoch update (fp64).

Follows the paper's statement of PPO (Sec. 2.1, Sec. 3) with the clipped
surrogate of Schulman et al. 2017, a clipped value loss, an entropy bonus,
global gradient-norm clipping and Adam.  Optional parts: symmetry augmentation
with a mirror loss (Sec. 2.2) and training of the RND predictor on the same
minibatch rows (Sec. 2.2).

Oracle code: test infrastructure only.
"""
from dataclasses import dataclass
import numpy as np

from . import mlp, gaussian, adam, rng, symmetry

STAT_NAMES = ("surrogate", "value_loss", "entropy", "kl", "grad_norm", "clip_frac", "mirror_loss", "rnd_loss")


@dataclass
class PPOConfig:
    clip: float = 0.2
    value_coef: float = 1.0
    entropy_coef: float = 0.01
    max_grad_norm: float = 1.0
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    adam_eps: float = 1e-8
    epochs: int = 5
    minibatches: int = 4
    use_clipped_value_loss: bool = True
    seed: int = 0
    call_index: int = 0
    epoch_offset: int = 0
    elu_alpha: float = 1.0


@dataclass
class SymSpec:
    perm_obs_a: np.ndarray
    sign_obs_a: np.ndarray
    perm_obs_c: np.ndarray
    sign_obs_c: np.ndarray
    perm_act: np.ndarray
    sign_act: np.ndarray
    mirror_loss_coef: float = 1.0


def act(actor_flat, critic_flat, dims_a, dims_c, obs_a, obs_c, eps, alpha=1.0):
    """One rollout step: mu = actor(obs_a), V = critic(obs_c), a = mu + sigma*eps, log-density of a."""
    layers_a, log_std = mlp.unpack(actor_flat, dims_a, log_std=True)
    layers_c = mlp.unpack(critic_flat, dims_c)
    mu, _ = mlp.forward(layers_a, obs_a, alpha)
    V, _ = mlp.forward(layers_c, obs_c, alpha)
    sigma = np.broadcast_to(np.exp(log_std), mu.shape).copy()
    a = mu + sigma * np.asarray(eps, np.float64)
    return dict(actions=a, logp=gaussian.log_prob(a, mu, sigma), values=V[:, 0], mu=mu, sigma=sigma)


def minibatch_loss_and_grads(actor_flat, critic_flat, dims_a, dims_c, batch, cfg, sym=None, input_grads=False,
                             sides=None, per_row=False):
    """Loss terms and flat gradients for one minibatch.

    batch: dict of row-gathered arrays obs_a, obs_c, actions, logp, adv, returns,
    values, mu, sigma (the last five are the rollout's recorded "old" quantities).
    With `sym`, the mb rows are followed by their mirrored copies (observations
    and actions mirrored; advantages, returns, old values, old log-densities
    copied) and every mean runs over the 2*mb rows.
    With input_grads the derivatives of the loss w.r.t. obs_a and obs_c are returned as well (a recurrent
    memory in front of the networks needs them).

    The clipped surrogate and the clipped value loss have a kink where the ratio (the value change) meets the
    clip range; there both one-sided derivatives are sub-gradients, and which one an implementation takes for a
    row that sits on the kink to within rounding is decided by its rounding.  `sides` lets a caller evaluate the
    other one: dict(policy={row: bool}, value={row: bool}) replaces, for the listed rows of this minibatch
    (mirrored copies count from mb), the predicate "inside the clip range" by the given truth value.  The loss
    terms do not depend on it (they are continuous); the gradient and the clip fraction do.  With per_row the
    returned terms also hold the per-row ratio, new value and the two predicates.
    """
    alpha = cfg.elu_alpha
    layers_a, log_std = mlp.unpack(actor_flat, dims_a, log_std=True)
    layers_c = mlp.unpack(critic_flat, dims_c)
    f64 = lambda k: np.asarray(batch[k], np.float64)
    obs_a, obs_c, actions = f64("obs_a"), f64("obs_c"), f64("actions")
    logp_old, adv, ret, v_old = f64("logp"), f64("adv"), f64("returns"), f64("values")
    mb = obs_a.shape[0]
    if sym is not None:
        obs_a = np.concatenate([obs_a, symmetry.mirror(obs_a, sym.perm_obs_a, sym.sign_obs_a)])
        obs_c = np.concatenate([obs_c, symmetry.mirror(obs_c, sym.perm_obs_c, sym.sign_obs_c)])
        actions = np.concatenate([actions, symmetry.mirror(actions, sym.perm_act, sym.sign_act)])
        logp_old, adv, ret, v_old = (np.concatenate([v, v]) for v in (logp_old, adv, ret, v_old))
    n = obs_a.shape[0]

    mu, cache_a = mlp.forward(layers_a, obs_a, alpha)
    Vout, cache_c = mlp.forward(layers_c, obs_c, alpha)
    V = Vout[:, 0]
    sigma = np.exp(log_std)
    zs = (actions - mu) / sigma
    logp = gaussian.log_prob(actions, mu, np.broadcast_to(sigma, mu.shape))
    H = gaussian.entropy(sigma)

    ratio = np.exp(logp - logp_old)
    ratio_c = np.clip(ratio, 1.0 - cfg.clip, 1.0 + cfg.clip)
    s1, s2 = -adv * ratio, -adv * ratio_c
    surrogate = np.mean(np.maximum(s1, s2))
    in_range = (ratio >= 1.0 - cfg.clip) & (ratio <= 1.0 + cfg.clip)
    active = in_range | (s1 >= s2)                                  # clipped branch is flat in ratio outside the range
    for r, side in ((sides or {}).get("policy") or {}).items():
        # outside the range the unclipped term is the larger one iff moving further out raises -A*ratio
        upper = abs(ratio[r] - (1.0 + cfg.clip)) <= abs(ratio[r] - (1.0 - cfg.clip))
        in_range[r] = side
        active[r] = side or (adv[r] < 0.0 if upper else adv[r] > 0.0)
    d_ratio = np.where(active, -adv, 0.0) / n

    if cfg.use_clipped_value_loss:
        v_clip = v_old + np.clip(V - v_old, -cfg.clip, cfg.clip)
        e1, e2 = (V - ret) ** 2, (v_clip - ret) ** 2
        value_loss = np.mean(np.maximum(e1, e2))
        # the clipped branch is flat in V only where the clamp is active; inside the clip range V_clip == V
        v_in_range = np.abs(V - v_old) <= cfg.clip
        v_active = v_in_range | (e1 >= e2)
        for r, side in ((sides or {}).get("value") or {}).items():
            # outside the range the unclipped square is the larger one iff V moves away from the return
            v_in_range[r] = side
            v_active[r] = side or ((V[r] - ret[r]) * (V[r] - v_old[r]) > 0.0)
        dV = np.where(v_active, 2.0 * (V - ret), 0.0) / n
    else:
        value_loss = np.mean((ret - V) ** 2)
        v_in_range = np.ones(n, bool)
        dV = 2.0 * (V - ret) / n

    d_logp = d_ratio * ratio
    d_mu = d_logp[:, None] * zs / sigma
    d_log_std = np.sum(d_logp[:, None] * (zs ** 2 - 1.0), axis=0) - cfg.entropy_coef * np.ones_like(sigma)

    loss = surrogate + cfg.value_coef * value_loss - cfg.entropy_coef * H
    mirror_l = 0.0
    if sym is not None:
        mirror_l, d_mirror = symmetry.mirror_loss(mu[:mb], mu[mb:], sym.perm_act, sym.sign_act)
        d_mu[mb:] += sym.mirror_loss_coef * d_mirror
        loss += sym.mirror_loss_coef * mirror_l

    grads_a, dx_a = mlp.backward(layers_a, cache_a, d_mu, alpha)
    grads_c, dx_c = mlp.backward(layers_c, cache_c, (cfg.value_coef * dV)[:, None], alpha)
    g_actor = mlp.pack(grads_a, d_log_std)
    g_critic = mlp.pack(grads_c)

    mu_old, sigma_old = f64("mu"), f64("sigma")
    kl = np.mean(gaussian.kl_old_new(mu_old, sigma_old, mu[:mb], np.broadcast_to(sigma, mu_old.shape)))
    terms = dict(loss=float(loss), surrogate=float(surrogate), value_loss=float(value_loss), entropy=float(H),
                 kl=float(kl), clip_frac=float(np.mean(~in_range)), mirror_loss=float(mirror_l))
    if per_row:
        terms.update(ratio=ratio, V=V, in_range=in_range, v_in_range=v_in_range, adv=adv)
    if input_grads:
        return terms, g_actor, g_critic, dx_a, dx_c
    return terms, g_actor, g_critic


def rnd_predictor_loss_and_grad(pred_flat, targ_flat, dims, x, alpha=1.0):
    """mean over rows and embedding dims of (pred(x) - target(x))^2, gradient w.r.t. the predictor."""
    lp, lt = mlp.unpack(pred_flat, dims), mlp.unpack(targ_flat, dims)
    yp, cache = mlp.forward(lp, x, alpha)
    yt, _ = mlp.forward(lt, x, alpha)
    diff = yp - yt
    grads, _ = mlp.backward(lp, cache, 2.0 * diff / diff.size, alpha)
    return float(np.mean(diff ** 2)), mlp.pack(grads)


def optimiser_step(actor, critic, dims_a, dims_c, batch, cfg, opt, sym=None, rnd=None, sides=None, per_row=False):
    """One optimiser step on one minibatch: loss and gradients, global gradient-norm clip, Adam on actor and
    critic with the shared step counter, then (with rnd) one Adam step of the RND predictor on the same rows.

    opt and rnd are updated in place (their arrays are replaced, not written into).  Returns
    (actor, critic, terms, g_actor, g_critic, grad_norm, rnd_loss).
    """
    terms, g_a, g_c = minibatch_loss_and_grads(actor, critic, dims_a, dims_c, batch, cfg, sym, sides=sides, per_row=per_row)
    norm = adam.global_norm([g_a, g_c])
    s = adam.clip_scale(norm, cfg.max_grad_norm)
    t0 = opt["step"]
    actor, opt["m_a"], opt["v_a"], _ = adam.adam_step(actor, s * g_a, opt["m_a"], opt["v_a"], t0, cfg.lr, cfg.beta1, cfg.beta2, cfg.adam_eps)
    critic, opt["m_c"], opt["v_c"], opt["step"] = adam.adam_step(critic, s * g_c, opt["m_c"], opt["v_c"], t0, cfg.lr, cfg.beta1, cfg.beta2, cfg.adam_eps)
    rnd_loss = 0.0
    if rnd is not None:
        x = np.asarray(batch["obs_a"], np.float64)
        if rnd.get("subset") is not None:
            x = x[:, np.asarray(rnd["subset"])]
        rnd_loss, g_p = rnd_predictor_loss_and_grad(rnd["pred"], rnd["targ"], rnd["dims"], x, cfg.elu_alpha)
        rnd["pred"], rnd["m"], rnd["v"], rnd["step"] = adam.adam_step(
            rnd["pred"], g_p, rnd["m"], rnd["v"], rnd["step"], rnd.get("lr", cfg.lr), cfg.beta1, cfg.beta2, cfg.adam_eps)
        rnd["g"] = g_p
    return actor, critic, terms, g_a, g_c, norm, rnd_loss


def copy_state(actor, critic, opt, rnd):
    """Deep copy of everything an optimiser step changes."""
    return dict(actor=actor.copy(), critic=critic.copy(), opt={k: (v.copy() if k != "step" else v) for k, v in opt.items()},
                rnd=None if rnd is None else {k: (np.copy(v) if k in ("pred", "m", "v") else v) for k, v in rnd.items()})


def ppo_update(actor, critic, dims_a, dims_c, rollout, cfg, opt, sym=None, rnd=None, record=False, sides=None):
    """E epochs x M minibatches over the flattened [T*N] rollout.

    actor/critic: flat parameter vectors.  opt: dict with m_a, v_a, m_c, v_c (flat
    Adam moments) and step (shared counter).  rollout: dict of arrays with B = T*N
    leading rows (flat index b = t*N + n).  rnd: optional dict with
    pred, targ (flat), dims, subset (column indices or None), m, v, step, lr.
    Returns dict(actor, critic, opt, stats[E*M, 8], g_actor, g_critic, rnd, perms); with record=True also
    `trace`: per optimiser step the state before it, its gradients, the state after it and the per-row ratio,
    new value, clip predicates and advantages of its minibatch.
    sides: optional {optimiser step index within this call: sides dict of minibatch_loss_and_grads}.
    """
    actor = np.asarray(actor, np.float64).copy(); critic = np.asarray(critic, np.float64).copy()
    opt = {k: (np.asarray(v, np.float64).copy() if k != "step" else int(v)) for k, v in opt.items()}
    flat = {k: np.asarray(v) for k, v in rollout.items()}
    B = flat["logp"].shape[0]
    for k in flat:
        assert flat[k].shape[0] == B, (k, flat[k].shape, B)
    assert B % cfg.minibatches == 0
    mb = B // cfg.minibatches
    if rnd is not None:
        rnd = dict(rnd); rnd["pred"] = np.asarray(rnd["pred"], np.float64).copy()
        rnd["m"] = np.asarray(rnd["m"], np.float64).copy(); rnd["v"] = np.asarray(rnd["v"], np.float64).copy()
    stats, perms, trace = [], [], []
    g_a = g_c = None
    for e in range(cfg.epochs):
        perm = rng.permutation(cfg.seed, cfg.call_index, e + cfg.epoch_offset, B)
        perms.append(perm)
        for m in range(cfg.minibatches):
            I = perm[m * mb:(m + 1) * mb]
            batch = {k: v[I] for k, v in flat.items()}
            before = copy_state(actor, critic, opt, rnd) if record else None
            actor, critic, terms, g_a, g_c, norm, rnd_loss = optimiser_step(
                actor, critic, dims_a, dims_c, batch, cfg, opt, sym, rnd, (sides or {}).get(e * cfg.minibatches + m), per_row=record)
            if record:
                trace.append(dict(rows=I, before=before, g_actor=g_a, g_critic=g_c, actor=actor.copy(), critic=critic.copy(),
                                  g_pred=None if rnd is None else rnd["g"], pred=None if rnd is None else rnd["pred"].copy(),
                                  opt={k: (v.copy() if k != "step" else v) for k, v in opt.items()},
                                  per_row={k: terms[k] for k in ("ratio", "V", "in_range", "v_in_range", "adv")}))
            stats.append([terms["surrogate"], terms["value_loss"], terms["entropy"], terms["kl"], norm,
                          terms["clip_frac"], terms["mirror_loss"], rnd_loss])
    return dict(actor=actor, critic=critic, opt=opt, stats=np.array(stats), g_actor=g_a, g_critic=g_c,
                rnd=rnd, perms=np.array(perms), trace=trace)
