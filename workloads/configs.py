"""Workload definitions and seeded input generators.

Simulator roll-outs are replaced by seeded tensors with the stated shapes and
distributions.  All draws come from numpy.random.Generator(PCG64(seed)); arrays
are float32 / uint8 / int32 exactly as they are handed to either implementation.
"""
from dataclasses import dataclass, field, replace
import numpy as np

MASTER_SEED = 20250910


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    N: int
    T: int
    Da: int
    Dc: int
    A: int
    hidden: tuple
    epochs: int = 5
    minibatches: int = 4
    gamma: float = 0.99
    lam: float = 0.95
    clip: float = 0.2
    value_coef: float = 1.0
    entropy_coef: float = 0.01
    max_grad_norm: float = 1.0
    lr: float = 1e-3
    reward_mean: float = 0.5
    reward_std: float = 0.3
    done_p: float = 1e-3
    heavy_tail: bool = False
    height_scan: int = 0            # trailing obs columns ~ U(-1, 1)
    symmetry: bool = False
    mirror_loss_coef: float = 1.0
    bc: bool = False
    student_hidden: tuple = ()
    student_obs: int = 0
    student_noise: float = 0.05
    rnd: bool = False
    rnd_hidden: tuple = ()
    rnd_out: int = 0
    rnd_weight: float = 0.5
    rnd_subset: int = 0             # > 0: the RND networks read this many of the Da observation columns
    timeout_p: float = 0.0          # per-step probability that an episode ends by time limit (also sets done)
    memory_hidden: int = 0          # > 0: actor and critic each have a GRU memory of this width in front of their MLP
    student_memory: int = 0         # > 0: the distillation student has a memory of this width in front of its MLP
    memory_cell: str = "gru"        # "gru" or "lstm": the cell of every memory of the workload

    @property
    def B(self):
        return self.T * self.N

    @property
    def dims_actor(self):
        return (self.memory_hidden or self.Da,) + tuple(self.hidden) + (self.A,)

    @property
    def dims_critic(self):
        return (self.memory_hidden or self.Dc,) + tuple(self.hidden) + (1,)

    @property
    def dims_student(self):
        return (self.student_memory or self.student_obs,) + tuple(self.student_hidden) + (self.A,)

    @property
    def dims_rnd(self):
        return (self.rnd_subset or self.Da,) + tuple(self.rnd_hidden) + (self.rnd_out,)

    def scaled(self, N):
        """Same workload at another environment count (parity tests at oracle-friendly sizes)."""
        return replace(self, N=N)


WORKLOADS = {
    "tiny": Workload("tiny", 1, N=64, T=24, Da=48, Dc=48, A=12, hidden=(128, 128),
                     reward_mean=0.0, reward_std=0.1, done_p=0.02),
    "flat": Workload("flat", 2, N=4096, T=24, Da=48, Dc=48, A=12, hidden=(512, 256, 128), heavy_tail=True),
    "rough": Workload("rough", 3, N=4096, T=24, Da=235, Dc=235, A=12, hidden=(512, 256, 128),
                      height_scan=187, symmetry=True),
    "distill": Workload("distill", 4, N=4096, T=24, Da=235, Dc=235, A=12, hidden=(512, 256, 128),
                        height_scan=187, bc=True, student_hidden=(256, 256, 128), student_obs=48,
                        epochs=2, minibatches=4),
    "curiosity": Workload("curiosity", 5, N=16384, T=24, Da=48, Dc=48, A=12, hidden=(512, 256, 128),
                          heavy_tail=True, rnd=True, rnd_hidden=(256, 256), rnd_out=64, minibatches=8),
    # the two variants below exercise paths the five configurations above leave cold: episodes cut by a time limit
    # (value bootstrap through the reward) next to early terminations, and RND on a strict subset of the state
    "flat_timeouts": Workload("flat_timeouts", 6, N=4096, T=24, Da=48, Dc=48, A=12, hidden=(512, 256, 128),
                              heavy_tail=True, done_p=0.01, timeout_p=0.02),
    "curiosity_subset": Workload("curiosity_subset", 7, N=16384, T=24, Da=48, Dc=48, A=12, hidden=(512, 256, 128),
                                 heavy_tail=True, rnd=True, rnd_hidden=(256, 256), rnd_out=64, minibatches=8,
                                 rnd_subset=24),
    # recurrent actor-critic: a 256-wide GRU (or, with memory_cell="lstm", LSTM) memory per network, episodes end
    # often enough that every roll-out holds resets
    "recurrent": Workload("recurrent", 8, N=4096, T=24, Da=48, Dc=48, A=12, hidden=(512, 256, 128), heavy_tail=True,
                          done_p=0.01, memory_hidden=256),
    "recurrent_lstm": Workload("recurrent_lstm", 10, N=4096, T=24, Da=48, Dc=48, A=12, hidden=(512, 256, 128),
                               heavy_tail=True, done_p=0.01, memory_hidden=256, memory_cell="lstm"),
    # distillation into a recurrent student: the distill workload's teacher, a student with a 256-wide GRU memory
    "distill_recurrent": Workload("distill_recurrent", 9, N=4096, T=24, Da=235, Dc=235, A=12, hidden=(512, 256, 128),
                                  height_scan=187, bc=True, student_hidden=(256, 128), student_obs=48, epochs=2,
                                  minibatches=4, done_p=0.01, student_memory=256),
}


def xavier_mlp(gen, dims, log_std=False):
    """Flat float32 parameters: per layer W [in, out] row-major ~ U(-a, a), a = sqrt(6/(in+out)), then b = 0;
    an actor's buffer ends with log_std = 0."""
    parts = []
    for i, o in zip(dims[:-1], dims[1:]):
        a = np.sqrt(6.0 / (i + o))
        parts.append(gen.uniform(-a, a, size=(i, o)).astype(np.float32).ravel())
        parts.append(np.zeros(o, np.float32))
    if log_std:
        parts.append(np.zeros(dims[-1], np.float32))
    return np.concatenate(parts)


def uniform_memory(gen, D, H, gates=3):
    """Flat float32 parameters of a recurrent cell with `gates` gates (GRU 3, LSTM 4): W_ih [D, G H], b_ih [G H],
    W_hh [H, G H], b_hh [G H], all ~ U(-1/sqrt(H), 1/sqrt(H))."""
    a = 1.0 / np.sqrt(H)
    return gen.uniform(-a, a, size=gates * H * (D + H + 2)).astype(np.float32)


def random_involution(gen, n, p_fixed=0.2):
    """Random signed permutation (perm int32, sign float32) with mirror(mirror(x)) = x:
    indices are paired at random (a fraction stays fixed); both members of a pair share one sign."""
    idx = gen.permutation(n)
    n_fixed = int(round(p_fixed * n))
    if (n - n_fixed) % 2:
        n_fixed += 1
    perm = np.arange(n, dtype=np.int32)
    sign = np.ones(n, np.float32)
    for j in idx[:n_fixed]:
        sign[j] = gen.choice([-1.0, 1.0])
    rest = idx[n_fixed:]
    for a, b in zip(rest[0::2], rest[1::2]):
        perm[a], perm[b] = b, a
        sign[a] = sign[b] = gen.choice([-1.0, 1.0])
    return perm, sign


def _mirror_map_obs(gen, w):
    """Proprioceptive block in 12-wide groups, height scan as a 17 x 11 grid with the short axis reversed."""
    n_prop = w.Da - w.height_scan
    perm = np.arange(w.Da, dtype=np.int32)
    sign = np.ones(w.Da, np.float32)
    for g0 in range(0, n_prop, 12):
        g1 = min(g0 + 12, n_prop)
        p, s = random_involution(gen, g1 - g0)
        perm[g0:g1] = g0 + p
        sign[g0:g1] = s
    if w.height_scan:
        assert w.height_scan == 17 * 11
        grid = np.arange(w.height_scan).reshape(17, 11)[:, ::-1].ravel()
        perm[n_prop:] = n_prop + grid
    return perm, sign


def make_inputs(w, seed=None):
    """All seeded arrays of one workload.

    obs        [T+1, N, Da] float32 (slab T feeds the bootstrap value); the critic reads the same tensor
    rewards    [T, N] float32, dones [T, N] uint8 (timeouts [T, N] uint8, a subset of dones, if the workload has them)
    actor/critic/...  flat float32 parameter vectors
    """
    gen = np.random.Generator(np.random.PCG64(MASTER_SEED + w.cfg_id if seed is None else seed))
    T, N = w.T, w.N
    n_prop = w.Da - w.height_scan
    obs = gen.standard_normal((T + 1, N, n_prop), dtype=np.float32)
    if w.heavy_tail:
        obs = np.where(gen.random((T + 1, N, n_prop)) < 0.05, obs * 10.0, obs).astype(np.float32)
    if w.height_scan:
        scan = gen.uniform(-1.0, 1.0, size=(T + 1, N, w.height_scan)).astype(np.float32)
        obs = np.concatenate([obs, scan], axis=2)
    out = dict(
        obs=np.ascontiguousarray(obs),
        rewards=(w.reward_mean + w.reward_std * gen.standard_normal((T, N))).astype(np.float32),
        dones=(gen.random((T, N)) < w.done_p).astype(np.uint8),
        actor=xavier_mlp(gen, w.dims_actor, log_std=True),
        critic=xavier_mlp(gen, w.dims_critic),
    )
    if w.symmetry:
        po, so = _mirror_map_obs(gen, w)
        pa, sa = random_involution(gen, w.A)
        out.update(perm_obs=po, sign_obs=so, perm_act=pa, sign_act=sa)
    if w.bc:
        noise = (w.student_noise * gen.standard_normal((T, N, w.student_obs))).astype(np.float32)
        out["obs_student"] = np.ascontiguousarray(obs[:T, :, :w.student_obs] + noise)
        out["teacher"] = xavier_mlp(gen, w.dims_actor)
        out["student"] = xavier_mlp(gen, w.dims_student)
        if w.student_memory:
            lstm = w.memory_cell == "lstm"
            out["mem_student"] = uniform_memory(gen, w.student_obs, w.student_memory, 4 if lstm else 3)
            out["h_student"] = (0.5 * gen.standard_normal((N, (2 if lstm else 1) * w.student_memory))).astype(np.float32)
            out["reset0"] = (gen.random(N) < w.done_p).astype(np.uint8)
    if w.rnd:
        if w.rnd_subset:
            out["rnd_subset_idx"] = np.sort(gen.choice(w.Da, size=w.rnd_subset, replace=False)).astype(np.int32)
        out["rnd_target"] = xavier_mlp(gen, w.dims_rnd)
        out["rnd_predictor"] = xavier_mlp(gen, w.dims_rnd)
    if w.memory_hidden:
        H, lstm = w.memory_hidden, w.memory_cell == "lstm"
        G, S = (4, 2 * H) if lstm else (3, H)                      # gates, packed state width ([h | c] for the LSTM)
        out["mem_actor"], out["mem_critic"] = uniform_memory(gen, w.Da, H, G), uniform_memory(gen, w.Dc, H, G)
        out["h_actor"] = (0.5 * gen.standard_normal((N, S))).astype(np.float32)     # states carried in from before
        out["h_critic"] = (0.5 * gen.standard_normal((N, S))).astype(np.float32)
        out["reset0"] = (gen.random(N) < w.done_p).astype(np.uint8)                  # episode ends of the step before
    if w.timeout_p > 0.0:
        out["timeouts"] = (gen.random((T, N)) < w.timeout_p).astype(np.uint8)
        out["dones"] = out["dones"] | out["timeouts"]
    return out
