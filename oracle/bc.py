"""DAgger-style behaviour cloning update (fp64).

Sec. 2.1: data gathered by rolling out the student are relabelled with the
expert's actions and the student is trained on them by supervised regression.
Here the data are given; the update regresses the student's mean action on the
frozen teacher's mean action:

    target_b = teacher(obs_teacher_b)            (once)
    L = mean over rows and action dims of (student(obs_student) - target)^2

Oracle code: test infrastructure only.
"""
from dataclasses import dataclass
import numpy as np

from . import mlp, adam, rng


@dataclass
class BCConfig:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    adam_eps: float = 1e-8
    epochs: int = 2
    minibatches: int = 4
    max_grad_norm: float = 0.0      # <= 0: no clipping
    seed: int = 0
    call_index: int = 0
    epoch_offset: int = 0
    elu_alpha: float = 1.0


def teacher_targets(teacher_flat, dims_t, obs_teacher, alpha=1.0):
    out, _ = mlp.forward(mlp.unpack(teacher_flat, dims_t), obs_teacher, alpha)
    return out


def collect_step(student_flat, dims_s, teacher_flat, dims_t, obs_student, obs_teacher, alpha=1.0):
    """One collection step of the loop of Sec. 2.1: the student's (mean) action on its own observations, which
    drives the roll-out, and the expert's action on the same states, which becomes the regression target."""
    actions, _ = mlp.forward(mlp.unpack(student_flat, dims_s), obs_student, alpha)
    return actions, teacher_targets(teacher_flat, dims_t, obs_teacher, alpha)


def bc_loss_and_grad(student_flat, dims_s, obs_student, targets, alpha=1.0):
    layers = mlp.unpack(student_flat, dims_s)
    y, cache = mlp.forward(layers, obs_student, alpha)
    diff = y - np.asarray(targets, np.float64)
    grads, _ = mlp.backward(layers, cache, 2.0 * diff / diff.size, alpha)
    return float(np.mean(diff ** 2)), mlp.pack(grads)


def bc_update(student, dims_s, obs_student, targets, cfg, opt):
    """opt: dict m, v, step.  Returns dict(student, opt, stats[E*M, 2] = (loss, grad_norm), g, perms)."""
    student = np.asarray(student, np.float64).copy()
    m = np.asarray(opt["m"], np.float64).copy(); v = np.asarray(opt["v"], np.float64).copy(); step = int(opt["step"])
    B = np.asarray(obs_student).shape[0]
    assert B % cfg.minibatches == 0
    mb = B // cfg.minibatches
    stats, perms, g = [], [], None
    for e in range(cfg.epochs):
        perm = rng.permutation(cfg.seed, cfg.call_index, e + cfg.epoch_offset, B)
        perms.append(perm)
        for k in range(cfg.minibatches):
            I = perm[k * mb:(k + 1) * mb]
            loss, g = bc_loss_and_grad(student, dims_s, np.asarray(obs_student)[I], np.asarray(targets)[I], cfg.elu_alpha)
            norm = adam.global_norm([g])
            s = adam.clip_scale(norm, cfg.max_grad_norm)
            student, m, v, step = adam.adam_step(student, s * g, m, v, step, cfg.lr, cfg.beta1, cfg.beta2, cfg.adam_eps)
            stats.append([loss, norm])
    return dict(student=student, opt=dict(m=m, v=v, step=step), stats=np.array(stats), g=g, perms=np.array(perms))
