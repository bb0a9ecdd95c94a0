"""GPU parity of the distillation loop (paper Sec. 2.1): the collection step (student acts, expert relabels), the
update on device-resident counters, and the whole iteration recorded as a HIP graph and replayed."""
from dataclasses import replace
import numpy as np
import pytest
import torch

from oracle import bc as obc
from workloads import WORKLOADS, make_inputs, xavier_mlp
from gpu_util import dev, host, rel_l2, f32

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.fixture(scope="module")
def rx():
    import paper_2509_10771_amd as m
    m.rslx_device_check()
    return m


def _collect(rx, dims_s, dims_t, student, teacher, obs_s, obs_t):
    N, A = obs_s.shape[0], dims_s[-1]
    s, t = rx.Mlp(dims_s, dev(student)), rx.Mlp(dims_t, dev(teacher))
    actions, targets = torch.empty(N, A, device="cuda"), torch.empty(N, A, device="cuda")
    ws = rx.workspace(rx.rslx_bc_collect_workspace_bytes(s, t, N))
    rx.rslx_bc_collect(s, t, dev(obs_s), dev(obs_t), N, actions, targets, ws)
    torch.cuda.synchronize()
    return host(actions), host(targets)


@pytest.mark.parametrize("N", [1, 300, 4096])
def test_bc_collect_matches_oracle(rx, N):
    w = WORKLOADS["distill"].scaled(N)
    inp = make_inputs(w)
    a, t = _collect(rx, w.dims_student, w.dims_actor, inp["student"], inp["teacher"], inp["obs_student"][0], inp["obs"][0])
    a_ref, t_ref = obc.collect_step(inp["student"], w.dims_student, inp["teacher"], w.dims_actor, inp["obs_student"][0], inp["obs"][0])
    assert rel_l2(a, a_ref) <= 1e-5 and rel_l2(t, t_ref) <= 1e-5


def test_bc_collect_wide_layers_take_the_layered_path(rx):
    g = np.random.default_rng(2)
    ds, dt = (20, 640, 7), (33, 96, 1024, 7)
    student, teacher = xavier_mlp(g, ds), xavier_mlp(g, dt)
    xs, xt = g.standard_normal((77, 20), dtype=np.float32), g.standard_normal((77, 33), dtype=np.float32)
    a, t = _collect(rx, ds, dt, student, teacher, xs, xt)
    a_ref, t_ref = obc.collect_step(student, ds, teacher, dt, xs, xt)
    assert rel_l2(a, a_ref) <= 1e-5 and rel_l2(t, t_ref) <= 1e-5


def test_bc_collect_rejects_mismatched_action_widths(rx):
    g = np.random.default_rng(2)
    s, t = rx.Mlp((8, 16, 3), dev(xavier_mlp(g, (8, 16, 3)))), rx.Mlp((8, 16, 4), dev(xavier_mlp(g, (8, 16, 4))))
    x = torch.zeros(5, 8, device="cuda")
    out = torch.zeros(5, 4, device="cuda")
    with pytest.raises(rx.RslxError):
        rx.rslx_bc_collect(s, t, x, x, 5, out, out, rx.workspace(1 << 16))


def test_bc_update_dc_matches_oracle(rx):
    w = WORKLOADS["distill"].scaled(125)
    inp = make_inputs(w)
    B = w.B
    obs_t = inp["obs"][:w.T].reshape(B, -1); obs_s = inp["obs_student"].reshape(B, -1)
    tgt = obc.teacher_targets(inp["teacher"], w.dims_actor, obs_t).astype(np.float32)
    ns = inp["student"].size
    ocfg = obc.BCConfig(lr=f32(w.lr), beta1=f32(0.9), beta2=f32(0.999), adam_eps=f32(1e-8), epochs=2,
                        minibatches=w.minibatches, max_grad_norm=f32(0.5), seed=5, call_index=4)
    ref = obc.bc_update(inp["student"], w.dims_student, obs_s, tgt, ocfg, dict(m=np.zeros(ns), v=np.zeros(ns), step=0))
    student = rx.Mlp(w.dims_student, dev(inp["student"]), trainable=True)
    cfg = rx.BcCfg(lr=w.lr, epochs=2, minibatches=w.minibatches, max_grad_norm=0.5, seed=5, call_index=77)
    n = 2 * w.minibatches
    stats = torch.zeros(n, rx.NSTATS, device="cuda")
    ws = rx.workspace(rx.rslx_bc_update_workspace_bytes(student, None, B, cfg))
    ctr = rx.dev_counters(call_index=4)
    rx.rslx_bc_update_dc(student, None, dev(obs_s), None, dev(tgt), B, cfg, ctr, stats, ws)
    torch.cuda.synchronize()
    got = host(stats)
    assert abs(got[0, 0] - ref["stats"][0, 0]) <= TOL * ref["stats"][0, 0]
    assert abs(got[0, 4] - ref["stats"][0, 1]) <= TOL * ref["stats"][0, 1]
    assert rel_l2(host(student.params), ref["student"]) <= 2 * TOL
    assert host(ctr).tolist() == [0, 5, n, 0]


class DistillLoop:
    """T collection steps into the [T, N] buffers, then the update on the collected targets."""

    def __init__(self, rx, w, inp):
        self.rx, self.w = rx, w
        T, N, A = w.T, w.N, w.A
        self.student = rx.Mlp(w.dims_student, dev(inp["student"]), trainable=True)
        self.teacher = rx.Mlp(w.dims_actor, dev(inp["teacher"]))
        self.obs_s, self.obs_t = dev(inp["obs_student"]), dev(inp["obs"][:T])
        self.actions, self.targets = torch.zeros(T, N, A, device="cuda"), torch.zeros(T, N, A, device="cuda")
        self.cfg = rx.BcCfg(lr=w.lr, epochs=w.epochs, minibatches=w.minibatches, seed=21)
        self.stats = torch.zeros(w.epochs * w.minibatches, rx.NSTATS, device="cuda")
        self.cws = rx.workspace(rx.rslx_bc_collect_workspace_bytes(self.student, self.teacher, N))
        self.uws = rx.workspace(rx.rslx_bc_update_workspace_bytes(self.student, None, w.B, self.cfg))
        self.ctr = rx.dev_counters()
        self.state = [t.clone() for t in self.state_tensors()]

    def state_tensors(self):
        return [self.student.params, self.student.adam_m, self.student.adam_v, self.ctr]

    def reset(self):
        for t, t0 in zip(self.state_tensors(), self.state):
            t.copy_(t0)

    def outputs(self):
        return [self.actions, self.targets, self.stats, self.student.params, self.student.adam_v]

    def iterate(self):
        rx, w = self.rx, self.w
        for t in range(w.T):
            rx.rslx_bc_collect(self.student, self.teacher, self.obs_s[t], self.obs_t[t], w.N, self.actions[t],
                               self.targets[t], self.cws)
        rx.rslx_bc_update_dc(self.student, None, self.obs_s, None, self.targets, w.B, self.cfg, self.ctr, self.stats, self.uws)


def test_distillation_iteration_matches_oracle_and_graph_replays(rx):
    w = WORKLOADS["distill"].scaled(96)
    inp = make_inputs(w)
    T, B = w.T, w.B
    eager, rec = DistillLoop(rx, w, inp), DistillLoop(rx, w, inp)
    # oracle: the same loop, first iteration
    obs_s = inp["obs_student"].reshape(B, -1)
    a_ref, t_ref = [], []
    for t in range(T):
        a, tg = obc.collect_step(inp["student"], w.dims_student, inp["teacher"], w.dims_actor, inp["obs_student"][t], inp["obs"][t])
        a_ref.append(a); t_ref.append(tg)
    tgt = np.stack(t_ref).reshape(B, -1).astype(np.float32)
    ns = inp["student"].size
    ocfg = obc.BCConfig(lr=f32(w.lr), beta1=f32(0.9), beta2=f32(0.999), adam_eps=f32(1e-8), epochs=w.epochs,
                        minibatches=w.minibatches, max_grad_norm=0.0, seed=21, call_index=0)
    ref = obc.bc_update(inp["student"], w.dims_student, obs_s, tgt, ocfg, dict(m=np.zeros(ns), v=np.zeros(ns), step=0))

    rec.iterate()                     # first-use set-up of the kernels happens outside the recording
    torch.cuda.synchronize()
    assert rel_l2(host(rec.actions), np.stack(a_ref)) <= 1e-5 and rel_l2(host(rec.targets), np.stack(t_ref)) <= 1e-5
    assert abs(host(rec.stats)[0, 0] - ref["stats"][0, 0]) <= TOL * ref["stats"][0, 0]
    assert rel_l2(host(rec.student.params), ref["student"]) <= 2 * TOL
    rec.reset()
    for t in rec.outputs()[:3]:
        t.zero_()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rec.iterate()
    torch.cuda.synchronize()
    assert host(rec.ctr).tolist() == [0, 0, 0, 0]
    n = w.epochs * w.minibatches
    for k in range(3):
        g.replay()
        eager.iterate()
        torch.cuda.synchronize()
        for i, (tr, te) in enumerate(zip(rec.outputs(), eager.outputs())):
            assert torch.equal(tr, te), (k, i)
        assert host(rec.ctr).tolist() == [0, k + 1, (k + 1) * n, 0]


# ---- distillation into a recurrent student (GRU memory + MLP), paper Sec. 2.1 with Sec. 3 ----------------------
import ctypes as C
from oracle import recurrent as orec, gru as ogru


def _rec_flat(inp):
    return np.concatenate([inp["mem_student"], inp["student"]])


def _rec_student(rx, w, flat, opt=None):
    k = orec.CELLS[w.memory_cell].n_params(w.student_obs, w.student_memory)
    p = dev(flat, torch.float32)
    g = rx.Memory(rx.CELL_LSTM if w.memory_cell == "lstm" else rx.CELL_GRU, w.student_obs, w.student_memory, p[:k], trainable=True)
    m = rx.Mlp(w.dims_student, p[k:], trainable=True)
    if opt is not None:
        mm, vv = dev(opt["m"], torch.float32), dev(opt["v"], torch.float32)
        g.adam_m, g.adam_v, m.adam_m, m.adam_v = mm[:k], vv[:k], mm[k:], vv[k:]
    return g, m


def _rec_rollout(w, inp):
    """The oracle rolls the recurrent student over the T slabs; the teacher labels every visited state."""
    T, N = w.T, w.N
    flat = _rec_flat(inp)
    h, reset = inp["h_student"].astype(np.float64), inp["reset0"]
    acts, tgts, hs, h0 = [], [], [], None
    for t in range(T):
        a, h, hin = orec.bc_collect_step(flat, w.student_obs, w.student_memory, w.dims_student, inp["obs_student"][t], h, reset,
                                         cell=w.memory_cell)
        if t == 0:
            h0 = hin
        acts.append(a); hs.append(h)
        tgts.append(obc.teacher_targets(inp["teacher"], w.dims_actor, inp["obs"][t]))
        reset = inp["dones"][t]
    c32 = lambda x: np.ascontiguousarray(np.asarray(x, np.float32))
    return dict(actions=c32(np.stack(acts)), targets=c32(np.stack(tgts)), hs=c32(np.stack(hs)), h0=c32(h0))


@pytest.mark.parametrize("cell", ["gru", "lstm"])
@pytest.mark.parametrize("N", [96, 1000])
def test_recurrent_student_collection_matches_oracle(rx, N, cell):
    w = replace(WORKLOADS["distill_recurrent"].scaled(N), memory_cell=cell)
    inp = make_inputs(w)
    ref = _rec_rollout(w, inp)
    T, A, H = w.T, w.A, w.student_memory
    g, m = _rec_student(rx, w, _rec_flat(inp))
    teacher = rx.Mlp(w.dims_actor, dev(inp["teacher"]))
    S = inp["h_student"].shape[1]
    h, h0, h_dense = dev(inp["h_student"]), torch.zeros(N, S, device="cuda"), torch.zeros(N, H, device="cuda")
    obs_s, obs_t, dones, reset0 = dev(inp["obs_student"]), dev(inp["obs"]), dev(inp["dones"]), dev(inp["reset0"])
    actions, targets = torch.empty(T, N, A, device="cuda"), torch.empty(T, N, A, device="cuda")
    sws = rx.workspace(rx.rslx_memory_step_workspace_bytes(g, N))
    cws = rx.workspace(rx.rslx_bc_collect_workspace_bytes(m, teacher, N))
    for t in range(T):
        rx.rslx_memory_step(g, obs_s[t], N, h, reset0 if t == 0 else dones[t - 1], h0 if t == 0 else None, h_dense, sws)
        rx.rslx_bc_collect(m, teacher, h_dense, obs_t[t], N, actions[t], targets[t], cws)
        torch.cuda.synchronize()
        assert rel_l2(host(h), ref["hs"][t]) <= 2e-5, t
    assert rel_l2(host(actions), ref["actions"]) <= 2e-5 and rel_l2(host(targets), ref["targets"]) <= 1e-5
    assert rel_l2(host(h0), ref["h0"]) <= 1e-6


class RecDistillCase:
    def __init__(self, w, epochs, clip=0.0):
        self.w, self.epochs, self.clip = w, epochs, clip
        inp = self.inp = make_inputs(w)
        ro = _rec_rollout(w, inp)
        self.flat0 = _rec_flat(inp).astype(np.float32)
        self.oro = dict(obs=inp["obs_student"], targets=ro["targets"], dones=inp["dones"], h0=ro["h0"])
        self.ocfg = obc.BCConfig(lr=f32(w.lr), beta1=f32(0.9), beta2=f32(0.999), adam_eps=f32(1e-8), epochs=epochs,
                                 minibatches=w.minibatches, max_grad_norm=f32(clip), seed=5, call_index=2)
        n = self.flat0.size
        self.ref = orec.bc_update(self.flat0, w.student_obs, w.student_memory, w.dims_student, self.oro, self.ocfg,
                                  dict(m=np.zeros(n), v=np.zeros(n), step=0), record=True, cell=w.memory_cell)

    def run(self, rx, flat, opt, envs, epochs, minibatches, step0):
        w = self.w
        o = self.oro if envs is None else {k: (v[envs] if k == "h0" else v[:, envs]) for k, v in self.oro.items()}
        N = o["dones"].shape[1]
        g, m = _rec_student(rx, w, flat, opt)
        cfg = rx.BcCfg(lr=w.lr, epochs=epochs, minibatches=minibatches, max_grad_norm=self.clip, seed=5, call_index=2)
        stats = torch.zeros(epochs * minibatches, rx.NSTATS, device="cuda")
        ws = rx.workspace(rx.rslx_bc_update_recurrent_workspace_bytes(g, m, w.T, N, cfg))
        step = C.c_int64(step0)
        rx.rslx_bc_update_recurrent(g, m, dev(o["obs"]), dev(o["targets"]), dev(o["dones"]), dev(o["h0"]), w.T, N, cfg, step,
                                    stats, ws)
        torch.cuda.synchronize()
        params = np.concatenate([host(g.params), host(m.params)])
        grads = np.concatenate([host(g.grads), host(m.grads)])
        return host(stats), step.value, params, grads


def _check_rec_student(name, w, got, ref, tol):
    D, H = w.student_obs, w.student_memory
    C = orec.CELLS[w.memory_cell]
    G = C.GATES
    o = 0
    for nm, n in (("W_ih", D * G * H), ("b_ih", G * H), ("W_hh", H * G * H), ("b_hh", G * H), ("mlp", got.size - C.n_params(D, H))):
        r = np.asarray(ref[o:o + n], np.float64)
        err = np.linalg.norm(np.asarray(got[o:o + n], np.float64) - r)
        assert err <= tol * np.linalg.norm(r) + 1e-12, (name, nm, err, np.linalg.norm(r))
        o += n


@pytest.mark.parametrize("cell", ["gru", "lstm"])
@pytest.mark.parametrize("N,hidden,mem,clip", [(96, (64, 32), 32, 0.0), (140, (72, 40), 44, 0.5), (256, (256, 128), 256, 0.0)])
def test_bc_update_recurrent_matches_oracle(rx, N, hidden, mem, clip, cell):
    w = replace(WORKLOADS["distill_recurrent"].scaled(N), student_hidden=hidden, student_memory=mem, done_p=0.04, memory_cell=cell)
    case = RecDistillCase(w, 1, clip)
    ref = case.ref
    assert case.inp["dones"][:-1].sum() > 10
    # every optimiser step replayed from the oracle's state before it, on that minibatch's environment columns
    for k, tr in enumerate(ref["trace"]):
        b = tr["before"]
        stats, step, params, grads = case.run(rx, b["student"], b["opt"], tr["envs"], 1, 1, b["opt"]["step"])
        assert step == b["opt"]["step"] + 1
        assert abs(stats[0, 0] - ref["stats"][k, 0]) <= TOL * ref["stats"][k, 0]
        assert abs(stats[0, 4] - ref["stats"][k, 1]) <= TOL * ref["stats"][k, 1]
        _check_rec_student("g step %d" % k, w, grads, tr["g"], TOL)
        _check_rec_student("student step %d" % k, w, params, tr["student"], TOL)
    # one free-running call
    n = w.minibatches
    stats, step, params, _ = case.run(rx, case.flat0, None, None, 1, n, 0)
    assert step == n
    assert np.all(np.abs(stats[:, 0] - ref["stats"][:, 0]) <= 2e-2 * np.maximum(ref["stats"][:, 0], 1e-3))
    assert rel_l2(params, ref["student"]) <= 2 * TOL
