"""Recurrent actor-critic: act() with carried hidden states and the PPO update with back-propagation through
time (fp64).

Sec. 3 of the paper: recurrent networks are supported for the RL and the distillation setting by managing the
hidden states across roll-outs and back-propagating through time.  The model here: actor and critic each own a
memory, a GRU (oracle.gru) or an LSTM (oracle.lstm, `cell="lstm"`; its state is the packed pair [h | c] and the
MLP sees h), whose hidden state feeds their MLP (oracle.mlp),

    h^a_t = GRU_a(obs^a_t, hin^a_t),  mu_t = actor_mlp(h^a_t);    h^c_t = GRU_c(obs^c_t, hin^c_t),  V_t = critic_mlp(h^c_t)

Hidden-state management: the state is zeroed for an environment whose episode ended on the previous step, it
is carried from one roll-out into the next, and the roll-out stores the state it started from (h0, after any
reset) so that the update can re-run the sequence exactly.

Update: minibatches are sets of whole environment columns (all T steps of N / M environments, environments
shuffled per epoch); each is re-run through the memory from its stored h0 with the same resets, the PPO loss
(oracle.ppo.minibatch_loss_and_grads, means over the T * N / M samples) is back-propagated through the MLPs
into the hidden states and from there through time (truncated at the roll-out start, never across an episode
boundary).  One gradient norm over all four parameter sets, one Adam step counter.

Distillation with a recurrent student (Sec. 2.1 with Sec. 3): the student, a GRU memory in front of an MLP, is
rolled out with its state carried and reset like the actor's; the expert's actions on the visited states are the
targets; the update regresses the student's outputs on them over whole environment columns with the same
back-propagation through time (bc_* functions below).

A network's flat parameter vector is the GRU layout followed by the MLP layout (log_std last for the actor).

Oracle code: test infrastructure only.
"""
import numpy as np

from . import gru, lstm, mlp, adam, rng
from . import ppo as _ppo


CELLS = {"gru": gru, "lstm": lstm}     # same interface; the state is packed per row (GRU: h, LSTM: [h | c])


def split(flat, D, H, cell="gru"):
    """(memory part, mlp part) of a recurrent network's flat parameter vector."""
    k = CELLS[cell].n_params(D, H)
    flat = np.asarray(flat, np.float64)
    return flat[:k], flat[k:]


def act(actor, critic, D_a, D_c, H, dims_a, dims_c, obs_a, obs_c, h_a, h_c, reset, eps, alpha=1.0, cell="gru"):
    """One roll-out step.  reset [N] (0/1): environments whose episode ended on the previous step start from a
    zero state.  Returns the outputs of ppo.act plus the new states h_a, h_c and the states the step started
    from (hin_a, hin_c).  States are packed per row as the cell defines (GRU: h; LSTM: [h | c])."""
    C = CELLS[cell]
    ga, ma = split(actor, D_a, H, cell)
    gc, mc = split(critic, D_c, H, cell)
    keep = (1.0 - np.asarray(reset, np.float64))[:, None]
    hin_a, hin_c = np.asarray(h_a, np.float64) * keep, np.asarray(h_c, np.float64) * keep
    ha, _ = C.cell(C.unpack(ga, D_a, H), obs_a, hin_a)
    hc, _ = C.cell(C.unpack(gc, D_c, H), obs_c, hin_c)
    out = _ppo.act(ma, mc, dims_a, dims_c, C.hidden(ha, H), C.hidden(hc, H), eps, alpha)
    out.update(h_a=ha, h_c=hc, hin_a=hin_a, hin_c=hin_c)
    return out


def minibatch_loss_and_grads(actor, critic, D_a, D_c, H, dims_a, dims_c, batch, cfg, cell="gru"):
    """batch: arrays with leading [T, nb]: obs_a, obs_c, actions, logp, adv, returns, values, mu, sigma, dones,
    and h0_a, h0_c [nb, H].  Returns (terms, g_actor, g_critic) in the flat layouts."""
    C = CELLS[cell]
    ga, ma = split(actor, D_a, H, cell)
    gc, mc = split(critic, D_c, H, cell)
    pa, pc = C.unpack(ga, D_a, H), C.unpack(gc, D_c, H)
    dones = np.asarray(batch["dones"])
    T, nb = dones.shape
    Ha, cache_a = C.sequence_forward(pa, batch["obs_a"], batch["h0_a"], dones)
    Hc, cache_c = C.sequence_forward(pc, batch["obs_c"], batch["h0_c"], dones)
    rows = {k: np.asarray(batch[k]).reshape((T * nb,) + np.asarray(batch[k]).shape[2:])
            for k in ("actions", "logp", "adv", "returns", "values", "mu", "sigma")}
    rows["obs_a"], rows["obs_c"] = Ha.reshape(T * nb, H), Hc.reshape(T * nb, H)
    terms, g_ma, g_mc, dHa, dHc = _ppo.minibatch_loss_and_grads(ma, mc, dims_a, dims_c, rows, cfg, None, input_grads=True)
    g_ga, _ = C.sequence_backward(pa, cache_a, dones, dHa.reshape(T, nb, H))
    g_gc, _ = C.sequence_backward(pc, cache_c, dones, dHc.reshape(T, nb, H))
    return terms, np.concatenate([g_ga, g_ma]), np.concatenate([g_gc, g_mc])


def ppo_update(actor, critic, D_a, D_c, H, dims_a, dims_c, rollout, cfg, opt, record=False, cell="gru"):
    """E epochs x M minibatches of whole environment columns.

    rollout: arrays [T, N, ...] obs_a, obs_c, actions, logp, adv, returns, values, mu, sigma, dones and
    h0_a, h0_c [N, H].  opt: m_a, v_a, m_c, v_c, step.  Environment order of epoch e:
    rng.permutation(seed, call_index, e + epoch_offset, N); minibatch m takes the m-th contiguous slice.
    """
    actor = np.asarray(actor, np.float64).copy(); critic = np.asarray(critic, np.float64).copy()
    opt = {k: (np.asarray(v, np.float64).copy() if k != "step" else int(v)) for k, v in opt.items()}
    N = np.asarray(rollout["dones"]).shape[1]
    assert N % cfg.minibatches == 0
    nb = N // cfg.minibatches
    stats, perms, trace = [], [], []
    g_a = g_c = None
    for e in range(cfg.epochs):
        perm = rng.permutation(cfg.seed, cfg.call_index, e + cfg.epoch_offset, N)
        perms.append(perm)
        for m in range(cfg.minibatches):
            envs = perm[m * nb:(m + 1) * nb]
            batch = {k: (np.asarray(v)[envs] if k in ("h0_a", "h0_c") else np.asarray(v)[:, envs]) for k, v in rollout.items()}
            before = dict(actor=actor.copy(), critic=critic.copy(),
                          opt={k: (v.copy() if k != "step" else v) for k, v in opt.items()}) if record else None
            terms, g_a, g_c = minibatch_loss_and_grads(actor, critic, D_a, D_c, H, dims_a, dims_c, batch, cfg, cell)
            norm = adam.global_norm([g_a, g_c])
            s = adam.clip_scale(norm, cfg.max_grad_norm)
            t0 = opt["step"]
            actor, opt["m_a"], opt["v_a"], _ = adam.adam_step(actor, s * g_a, opt["m_a"], opt["v_a"], t0, cfg.lr, cfg.beta1, cfg.beta2, cfg.adam_eps)
            critic, opt["m_c"], opt["v_c"], opt["step"] = adam.adam_step(critic, s * g_c, opt["m_c"], opt["v_c"], t0, cfg.lr, cfg.beta1, cfg.beta2, cfg.adam_eps)
            if record:
                trace.append(dict(envs=envs, before=before, g_actor=g_a, g_critic=g_c, actor=actor.copy(), critic=critic.copy()))
            stats.append([terms["surrogate"], terms["value_loss"], terms["entropy"], terms["kl"], norm,
                          terms["clip_frac"], 0.0, 0.0])
    return dict(actor=actor, critic=critic, opt=opt, stats=np.array(stats), g_actor=g_a, g_critic=g_c,
                perms=np.array(perms), trace=trace)


def bc_collect_step(student, D, H, dims_s, obs_s, h, reset, alpha=1.0, cell="gru"):
    """One collection step of a recurrent student: (mean action, new state, state the step started from)."""
    C = CELLS[cell]
    g, m = split(student, D, H, cell)
    hin = np.asarray(h, np.float64) * (1.0 - np.asarray(reset, np.float64))[:, None]
    h_new, _ = C.cell(C.unpack(g, D, H), obs_s, hin)
    a, _ = mlp.forward(mlp.unpack(m, dims_s), C.hidden(h_new, H), alpha)
    return a, h_new, hin


def bc_minibatch_loss_and_grad(student, D, H, dims_s, batch, alpha=1.0, cell="gru"):
    """batch: obs [T, nb, D], targets [T, nb, A], dones [T, nb], h0 [nb, H].
    L = mean over the T * nb rows and the A action dims of (student - target)^2; returns (L, flat gradient)."""
    C = CELLS[cell]
    g, m = split(student, D, H, cell)
    pg, layers = C.unpack(g, D, H), mlp.unpack(m, dims_s)
    dones = np.asarray(batch["dones"])
    T, nb = dones.shape
    Hs, cache_g = C.sequence_forward(pg, batch["obs"], batch["h0"], dones)
    y, cache_m = mlp.forward(layers, Hs.reshape(T * nb, H), alpha)
    diff = y - np.asarray(batch["targets"], np.float64).reshape(T * nb, -1)
    grads_m, dH = mlp.backward(layers, cache_m, 2.0 * diff / diff.size, alpha)
    g_g, _ = C.sequence_backward(pg, cache_g, dones, dH.reshape(T, nb, H))
    return float(np.mean(diff ** 2)), np.concatenate([g_g, mlp.pack(grads_m)])


def bc_update(student, D, H, dims_s, rollout, cfg, opt, record=False, cell="gru"):
    """E epochs x M minibatches of whole environment columns; cfg is an oracle.bc.BCConfig.
    rollout: obs [T, N, D], targets [T, N, A], dones [T, N], h0 [N, H].  opt: m, v, step."""
    student = np.asarray(student, np.float64).copy()
    opt = {k: (np.asarray(v, np.float64).copy() if k != "step" else int(v)) for k, v in opt.items()}
    N = np.asarray(rollout["dones"]).shape[1]
    assert N % cfg.minibatches == 0
    nb = N // cfg.minibatches
    stats, trace = [], []
    g = None
    for e in range(cfg.epochs):
        perm = rng.permutation(cfg.seed, cfg.call_index, e + cfg.epoch_offset, N)
        for m in range(cfg.minibatches):
            envs = perm[m * nb:(m + 1) * nb]
            batch = {k: (np.asarray(v)[envs] if k == "h0" else np.asarray(v)[:, envs]) for k, v in rollout.items()}
            before = dict(student=student.copy(), opt={k: (v.copy() if k != "step" else v) for k, v in opt.items()}) if record else None
            loss, g = bc_minibatch_loss_and_grad(student, D, H, dims_s, batch, cfg.elu_alpha, cell)
            norm = adam.global_norm([g])
            s = adam.clip_scale(norm, cfg.max_grad_norm)
            student, opt["m"], opt["v"], opt["step"] = adam.adam_step(student, s * g, opt["m"], opt["v"], opt["step"], cfg.lr,
                                                                      cfg.beta1, cfg.beta2, cfg.adam_eps)
            if record:
                trace.append(dict(envs=envs, before=before, g=g, student=student.copy()))
            stats.append([loss, norm])
    return dict(student=student, opt=opt, stats=np.array(stats), g=g, trace=trace)
