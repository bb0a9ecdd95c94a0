"""Benchmark of the whole PPO hot path on one MI355X.

One step = one training iteration of the "flat" workload (N = 4096 environments, T = 24, obs 48, actions 12,
actor and critic [512, 256, 128]): T act() calls + the bootstrap value + GAE + the 5-epoch x 4-minibatch PPO
update, all inputs resident in HBM.  Prints ONE JSON line; `value` is transitions (T*N) per second of the
whole iteration.  The roofline entry is measured live with HIP events recorded by the library around its
matrix-core launches; the CPU baseline times the fp64 oracle on a bounded sample of the same workload.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_MFMA_PEAK_TFLOPS = 157.3
HBM_PEAK_GBS = 8000.0


def kernel_sources_hash():
    """sha256/16 of the HIP sources, the stamp the counter summaries under profiles/ carry."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2509_10771_amd", "csrc", "*.hip")) +
                    glob.glob(os.path.join(ROOT, "paper_2509_10771_amd", "csrc", "*.h"))):
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def hbm_traffic_per_launch(workload, site):
    """HBM bytes per launch of a matrix-core launch site, from the rocprofv3 FETCH_SIZE / WRITE_SIZE summary of
    this workload under profiles/ (calibrated there against a kernel of known size).  None when there is no
    summary, when it was taken on other kernel sources than the ones in the tree, or when the site is not listed."""
    import re
    path = os.path.join(ROOT, "profiles", "%s_iteration_hbm_traffic.txt" % workload)
    if not os.path.exists(path):
        return None
    text = open(path).read()
    m = re.search(r"kernel sources sha256/16: ([0-9a-f]{16})", text)
    if not m or m.group(1) != kernel_sources_hash():
        return None
    m = re.match(r"gemm_dwdx_(\d+)x(\d+)_(\d+)x(\d+)$", site)
    if m:
        pat = r"gemm_pair_kernel<%s, %s, \d+, \d+, %s, %s, " % m.groups()
    else:
        m = re.match(r"gemm_(fwd|dx|dw)_(\d+)x(\d+)$", site)
        if not m:
            return None
        pat = r"gemm_kernel<%d, %s, %s, " % ({"fwd": 0, "dx": 1, "dw": 2}[m.group(1)], m.group(2), m.group(3))
    calls = total = 0.0
    for line in text.splitlines():
        if re.match(pat, line):
            f = line.split()
            calls += float(f[-4]); total += float(f[-4]) * float(f[-1]) * 1e6
    return total / calls if calls else None


def flops_per_sample_pass(dims_a, dims_c):
    """Forward + weight gradient + input gradient (none into the observations), 2 flops per multiply-add."""
    total = 0
    for dims in (dims_a, dims_c):
        for l, (i, o) in enumerate(zip(dims[:-1], dims[1:])):
            total += 2 * i * o * (3 if l > 0 else 2)
    return total


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="flat")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-trace", action="store_true", help="skip the per-launch HIP-event trace (no roofline entry)")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the same iteration")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU; run with --gpus 1 (environments are independent columns, so the path "
              "would shard by environment with one gradient all-reduce per optimiser step)")
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2509_10771_amd as rx
    from workloads import WORKLOADS, make_inputs

    rx.rslx_device_check()
    w = WORKLOADS[args.workload]
    inp = make_inputs(w)
    T, N, A, B = w.T, w.N, w.A, w.B
    dev = lambda x: torch.as_tensor(np.ascontiguousarray(x)).cuda()

    if w.bc:
        print(json.dumps(distill_iteration(args, rx, torch, np, w, inp)))
        return
    if w.memory_hidden:
        print(json.dumps(recurrent_iteration(args, rx, torch, np, w, inp)))
        return

    actor = rx.Mlp(w.dims_actor, dev(inp["actor"]), trainable=True, has_log_std=True)
    critic = rx.Mlp(w.dims_critic, dev(inp["critic"]), trainable=True)
    obs, rewards, dones = dev(inp["obs"]), dev(inp["rewards"]), dev(inp["dones"])
    timeouts = dev(inp["timeouts"]) if "timeouts" in inp else None
    rnd_sub = dev(inp["rnd_subset_idx"]) if "rnd_subset_idx" in inp else None
    actions, mu, sigma = (torch.empty(T, N, A, device="cuda") for _ in range(3))
    logp, values, adv, ret = (torch.empty(T, N, device="cuda") for _ in range(4))
    last = torch.empty(N, device="cuda")
    sym = rx.Sym(inp["perm_obs"], inp["sign_obs"], inp["perm_obs"], inp["sign_obs"], inp["perm_act"], inp["sign_act"],
                 w.mirror_loss_coef) if w.symmetry else None
    rnd = None
    if w.rnd:
        rnd_t = rx.Mlp(w.dims_rnd, dev(inp["rnd_target"]))
        rnd_p = rx.Mlp(w.dims_rnd, dev(inp["rnd_predictor"]), trainable=True)
        rnd = rx.RndTrain(rnd_t, rnd_p, subset_idx=rnd_sub, lr=w.lr)
        running = dev(np.array([0.0, 1.0, 1e-4], np.float32))
        r_int = torch.empty(N, device="cuda")
        rws = rx.workspace(rx.rslx_rnd_workspace_bytes(rnd_t, N))
        rew_work = torch.empty_like(rewards)
    rollout = rx.Rollout(T, N, obs[:T], obs[:T], actions, logp, values, mu, sigma, adv, ret)
    cfg_kw = dict(clip=w.clip, value_coef=w.value_coef, entropy_coef=w.entropy_coef, max_grad_norm=w.max_grad_norm,
                  lr=w.lr, epochs=w.epochs, minibatches=w.minibatches, seed=20250910)
    stats = torch.zeros(w.epochs * w.minibatches, rx.NSTATS, device="cuda")
    aws = rx.workspace(rx.rslx_act_workspace_bytes(actor, critic, N))
    gws = rx.workspace(rx.rslx_gae_workspace_bytes(T, N))
    uws = rx.workspace(rx.rslx_ppo_update_workspace_bytes(actor, critic, rollout, rx.PpoCfg(**cfg_kw), sym, rnd))
    adam_step = ctypes.c_int64(0)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    phase = {"act": [], "gae": [], "update": []}

    def step(it, timed):
        e = [ev() for _ in range(5)] if timed else None
        if timed:
            e[0].record()
        rew = rewards
        if w.rnd:
            rew_work.copy_(rewards)
            rew = rew_work
        for t in range(T):
            rx.rslx_act(actor, critic, obs[t], obs[t], N, 20250910, it * T + t, None, actions[t], logp[t], values[t],
                        mu[t], sigma[t], 0, aws)
            if w.rnd:
                rx.rslx_rnd(rnd_t, rnd_p, obs[t], N, w.Da, rnd_sub, w.dims_rnd[0], running, w.rnd_weight, 1, r_int, rew[t], rws)
        if timed:
            e[4].record()      # end of the T acting calls (env-steps are counted over these, not over the bootstrap)
        rx.rslx_act(None, critic, None, obs[T], N, 0, 0, None, None, None, last, None, None, rx.ACT_VALUES_ONLY, aws)
        if timed:
            e[1].record()
        rx.rslx_gae(rew, values, last, dones, timeouts, T, N, w.gamma, w.lam, 1, adv, ret, gws)
        if timed:
            e[2].record()
        rx.rslx_ppo_update(actor, critic, rollout, rx.PpoCfg(call_index=it, **cfg_kw), sym, rnd, adam_step, stats, uws)
        if timed:
            e[3].record()
        return e

    for it in range(args.warmup):
        step(it, False)
    torch.cuda.synchronize()
    # timed region: K whole iterations, no instrumentation inside the library
    t0 = time.perf_counter()
    evs = [step(args.warmup + it, True) for it in range(args.steps)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    phase["act_calls"] = []
    for e in evs:
        phase["act"].append(e[0].elapsed_time(e[1])); phase["gae"].append(e[1].elapsed_time(e[2]))
        phase["update"].append(e[2].elapsed_time(e[3])); phase["act_calls"].append(e[0].elapsed_time(e[4]))
    # the same K iterations again with the library's HIP-event trace on: per-kernel launch durations for the
    # roofline entry (two event records per launch cost ~10 % of throughput, so `value` comes from the run above)
    trace, traced_ms = [("untraced", 0.0, 0.0, 1.0)], None
    if not args.no_trace:
        rx.rslx_trace_begin(1 << 16)
        t2 = time.perf_counter()
        for it in range(args.steps):
            step(args.warmup + args.steps + it, False)
        torch.cuda.synchronize()
        traced_ms = (time.perf_counter() - t2) * 1e3 / args.steps
        trace = rx.rslx_trace_end()
    # the same iteration recorded once as a HIP graph (entry points on device-resident counters) and replayed K times
    graph_ms = None
    if not args.no_graph:
        ctr = rx.dev_counters(act_step=(args.warmup + 2 * args.steps) * T, call_index=args.warmup + 2 * args.steps,
                              adam_step=adam_step.value, rnd_adam_step=rnd.step.value if rnd else 0)

        def step_dc():
            rew = rewards
            if w.rnd:
                rew_work.copy_(rewards)
                rew = rew_work
            for t in range(T):
                rx.rslx_act_dc(actor, critic, obs[t], obs[t], N, 20250910, ctr, None, actions[t], logp[t], values[t],
                               mu[t], sigma[t], 0, aws)
                if w.rnd:
                    rx.rslx_rnd(rnd_t, rnd_p, obs[t], N, w.Da, rnd_sub, w.dims_rnd[0], running, w.rnd_weight, 1, r_int, rew[t], rws)
            rx.rslx_act_dc(None, critic, None, obs[T], N, 0, ctr, None, None, None, last, None, None, rx.ACT_VALUES_ONLY, aws)
            rx.rslx_gae(rew, values, last, dones, timeouts, T, N, w.gamma, w.lam, 1, adv, ret, gws)
            rx.rslx_ppo_update_dc(actor, critic, rollout, rx.PpoCfg(**cfg_kw), sym, rnd, ctr, stats, uws)

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step_dc()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t3) * 1e3 / args.steps
    med = {k: float(np.median(v)) for k, v in phase.items()}
    assert torch.isfinite(actor.params).all() and torch.isfinite(stats).all(), "training state became non-finite"

    roofline, breakdown = summarize_trace(trace, w, args.steps)

    sample_passes = w.epochs * B * (2 if w.symmetry else 1)
    upd_flops = flops_per_sample_pass(w.dims_actor, w.dims_critic) * sample_passes
    result = {
        "metric": "PPO update transitions/sec + act() env-steps/sec at 4096 envs, 1 GPU",
        "value": round(B / (ms_per_step * 1e-3), 1),
        "unit": "transitions/s (whole iteration: %d act + GAE + %dx%d PPO update)" % (T, w.epochs, w.minibatches),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: N=%d envs, T=%d, obs %d, act %d, actor/critic %s ELU, %d epochs x %d minibatches"
                   % (w.name, N, T, w.Da, A, list(w.hidden), w.epochs, w.minibatches)},
        "update_transitions_per_s": round(B / (med["update"] * 1e-3), 1),
        "update_sample_passes_per_s": round(sample_passes / (med["update"] * 1e-3), 1),
        "update_tflops": round(upd_flops / (med["update"] * 1e-3) / 1e12, 2),
        "act_env_steps_per_s": round(T * N / (med["act_calls"] * 1e-3), 1),
        "phase_ms": {k: round(v, 4) for k, v in med.items()},
        "traced_ms_per_step": None if traced_ms is None else round(traced_ms, 4),
        "graph_replay": None if graph_ms is None else {"ms_per_step": round(graph_ms, 4),
                                                       "value": round(B / (graph_ms * 1e-3), 1)},
        "roofline": roofline,
        "kernels": breakdown,
    }

    result["streaming"] = streaming_kernels(rx, torch, T, N, int(actor.params.numel() + critic.params.numel()))
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, inp)
    print(json.dumps(result))


def distill_iteration(args, rx, torch, np, w, inp):
    """One iteration of the distillation loop: T collection steps (student acts, teacher relabels) and the
    behaviour-cloning update on the collected targets."""
    T, N, A, B = w.T, w.N, w.A, w.B
    dev = lambda x: torch.as_tensor(np.ascontiguousarray(x)).cuda()
    student = rx.Mlp(w.dims_student, dev(inp["student"]), trainable=True)
    teacher = rx.Mlp(w.dims_actor, dev(inp["teacher"]))
    rec = w.student_memory > 0          # recurrent student: a GRU memory in front of the MLP, column-wise minibatches
    if rec:
        H = w.student_memory
        lstm = w.memory_cell == "lstm"
        gru = rx.Memory(rx.CELL_LSTM if lstm else rx.CELL_GRU, w.student_obs, H, dev(inp["mem_student"]), trainable=True)
        h, reset0, dones = dev(inp["h_student"]), dev(inp["reset0"]), dev(inp["dones"])
        h0, h_dense = torch.empty_like(h), torch.empty(N, H, device="cuda")
        sws = rx.workspace(rx.rslx_memory_step_workspace_bytes(gru, N))
    obs_s, obs_t = dev(inp["obs_student"]), dev(inp["obs"][:T])
    actions, targets = torch.empty(T, N, A, device="cuda"), torch.empty(T, N, A, device="cuda")
    cfg_kw = dict(lr=w.lr, epochs=w.epochs, minibatches=w.minibatches, seed=20250910)
    stats = torch.zeros(w.epochs * w.minibatches, rx.NSTATS, device="cuda")
    cws = rx.workspace(rx.rslx_bc_collect_workspace_bytes(student, teacher, N))
    uws = rx.workspace(rx.rslx_bc_update_recurrent_workspace_bytes(gru, student, T, N, rx.BcCfg(**cfg_kw)) if rec
                       else rx.rslx_bc_update_workspace_bytes(student, None, B, rx.BcCfg(**cfg_kw)))
    adam_step = ctypes.c_int64(0)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(it, timed, ctr=None):
        e = [ev() for _ in range(3)] if timed else None
        if timed:
            e[0].record()
        for t in range(T):
            if rec:
                reset = dones[t - 1] if t > 0 else (reset0 if it == 0 else dones[T - 1])
                rx.rslx_memory_step(gru, obs_s[t], N, h, reset, h0 if t == 0 else None, h_dense if lstm else None, sws)
                rx.rslx_bc_collect(student, teacher, h_dense if lstm else h, obs_t[t], N, actions[t], targets[t], cws)
            else:
                rx.rslx_bc_collect(student, teacher, obs_s[t], obs_t[t], N, actions[t], targets[t], cws)
        if timed:
            e[1].record()
        if rec:
            rx.rslx_bc_update_recurrent(gru, student, obs_s, targets, dones, h0, T, N, rx.BcCfg(call_index=it, **cfg_kw),
                                        adam_step, stats, uws)
        elif ctr is None:
            rx.rslx_bc_update(student, None, obs_s, None, targets, B, rx.BcCfg(call_index=it, **cfg_kw), adam_step, stats, uws)
        else:
            rx.rslx_bc_update_dc(student, None, obs_s, None, targets, B, rx.BcCfg(**cfg_kw), ctr, stats, uws)
        if timed:
            e[2].record()
        return e

    for it in range(args.warmup):
        step(it, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs = [step(args.warmup + it, True) for it in range(args.steps)]
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    med = {"collect": float(np.median([e[0].elapsed_time(e[1]) for e in evs])),
           "update": float(np.median([e[1].elapsed_time(e[2]) for e in evs]))}
    roofline, breakdown, traced_ms = None, None, None
    if not args.no_trace:
        rx.rslx_trace_begin(1 << 16)
        t2 = time.perf_counter()
        for it in range(args.steps):
            step(args.warmup + args.steps + it, False)
        torch.cuda.synchronize()
        traced_ms = (time.perf_counter() - t2) * 1e3 / args.steps
        roofline, breakdown = summarize_trace(rx.rslx_trace_end(), w, args.steps)
    graph_ms = None
    if not args.no_graph and not rec:
        ctr = rx.dev_counters(call_index=args.warmup + 2 * args.steps, adam_step=adam_step.value)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(0, False, ctr)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t3) * 1e3 / args.steps
    assert torch.isfinite(student.params).all() and torch.isfinite(stats).all(), "training state became non-finite"
    fwd = lambda dims: sum(2 * i * o for i, o in zip(dims[:-1], dims[1:]))
    upd_flops = (3 * fwd(w.dims_student) - 2 * w.dims_student[0] * w.dims_student[1]) * B * w.epochs
    col_flops = (fwd(w.dims_student) + fwd(w.dims_actor)) * B
    if rec:
        D = w.student_obs
        G = 4 if lstm else 3
        upd_flops = (3 * fwd(w.dims_student) + 2 * (D + H) * G * H + 2 * D * G * H + 4 * H * G * H) * B * w.epochs
        col_flops += 2 * (D + H) * G * H * B
    return {
        "metric": "BC (distillation) transitions/sec: collection (student acts, teacher relabels) + update, 1 GPU",
        "value": round(B / (ms_per_step * 1e-3), 1),
        "unit": "transitions/s (whole iteration: %d collect + %dx%d BC update)" % (T, w.epochs, w.minibatches),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: N=%d envs, T=%d, teacher %s, student %s%s ELU, %d epochs x %d minibatches"
                   % (w.name, N, T, list(w.dims_actor), "%s %d + MLP " % (w.memory_cell.upper(), w.student_memory) if rec else "", list(w.dims_student),
                      w.epochs, w.minibatches)},
        "phase_ms": {k: round(v, 4) for k, v in med.items()},
        "collect_tflops": round(col_flops / (med["collect"] * 1e-3) / 1e12, 2),
        "update_tflops": round(upd_flops / (med["update"] * 1e-3) / 1e12, 2),
        "traced_ms_per_step": None if traced_ms is None else round(traced_ms, 4),
        "graph_replay": None if graph_ms is None else {"ms_per_step": round(graph_ms, 4),
                                                       "value": round(B / (graph_ms * 1e-3), 1)},
        "roofline": roofline, "kernels": breakdown,
    }


def recurrent_iteration(args, rx, torch, np, w, inp):
    """One iteration with GRU memories: T recurrent act steps (states carried across iterations, reset at episode
    ends), bootstrap value, GAE, and the column-wise PPO update with back-propagation through time."""
    T, N, A, B, H = w.T, w.N, w.A, w.B, w.memory_hidden
    lstm = w.memory_cell == "lstm"
    G, S = (4, 2 * H) if lstm else (3, H)          # gates, packed state width
    dev = lambda x: torch.as_tensor(np.ascontiguousarray(x)).cuda()
    nets = []
    for which, D, dims, log_std in (("actor", w.Da, w.dims_actor, True), ("critic", w.Dc, w.dims_critic, False)):
        nets.append(rx.Memory(rx.CELL_LSTM if lstm else rx.CELL_GRU, D, H, dev(inp["mem_" + which]), trainable=True))
        nets.append(rx.Mlp(dims, dev(inp[which]), trainable=True, has_log_std=log_std))
    ga, ma, gc, mc = nets
    obs, rewards, dones = dev(inp["obs"]), dev(inp["rewards"]), dev(inp["dones"])
    h_a, h_c, reset0 = dev(inp["h_actor"]), dev(inp["h_critic"]), dev(inp["reset0"])
    h0_a, h0_c = torch.empty(N, S, device="cuda"), torch.empty(N, S, device="cuda")
    actions, mu, sigma = (torch.empty(T, N, A, device="cuda") for _ in range(3))
    logp, values, adv, ret = (torch.empty(T, N, device="cuda") for _ in range(4))
    last = torch.empty(N, device="cuda")
    rollout = rx.Rollout(T, N, obs[:T], obs[:T], actions, logp, values, mu, sigma, adv, ret)
    cfg_kw = dict(clip=w.clip, value_coef=w.value_coef, entropy_coef=w.entropy_coef, max_grad_norm=w.max_grad_norm,
                  lr=w.lr, epochs=w.epochs, minibatches=w.minibatches, seed=20250910)
    stats = torch.zeros(w.epochs * w.minibatches, rx.NSTATS, device="cuda")
    aws = rx.workspace(rx.rslx_act_recurrent_workspace_bytes(ga, ma, gc, mc, N))
    gws = rx.workspace(rx.rslx_gae_workspace_bytes(T, N))
    uws = rx.workspace(rx.rslx_ppo_update_recurrent_workspace_bytes(ga, ma, gc, mc, rollout, rx.PpoCfg(**cfg_kw)))
    adam_step = ctypes.c_int64(0)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(it, timed):
        e = [ev() for _ in range(5)] if timed else None
        if timed:
            e[0].record()
        for t in range(T):
            reset = dones[t - 1] if t > 0 else (reset0 if it == 0 else dones[T - 1])
            rx.rslx_act_recurrent(ga, ma, gc, mc, obs[t], obs[t], N, h_a, h_c, reset, h0_a if t == 0 else None,
                                  h0_c if t == 0 else None, 20250910, it * T + t, None, actions[t], logp[t], values[t], mu[t],
                                  sigma[t], 0, aws)
        if timed:
            e[4].record()      # end of the T acting calls
        rx.rslx_act_recurrent(None, None, gc, mc, None, obs[T], N, None, h_c, dones[T - 1], None, None, 0, 0, None, None, None,
                              last, None, None, rx.ACT_VALUES_ONLY, aws)
        if timed:
            e[1].record()
        rx.rslx_gae(rewards, values, last, dones, None, T, N, w.gamma, w.lam, 1, adv, ret, gws)
        if timed:
            e[2].record()
        rx.rslx_ppo_update_recurrent(ga, ma, gc, mc, rollout, dones, h0_a, h0_c, rx.PpoCfg(call_index=it, **cfg_kw), adam_step,
                                     stats, uws)
        if timed:
            e[3].record()
        return e

    for it in range(args.warmup):
        step(it, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs = [step(args.warmup + it, True) for it in range(args.steps)]
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    med = {k: float(np.median([e[i].elapsed_time(e[i + 1]) for e in evs])) for i, k in enumerate(("act", "gae", "update"))}
    med["act_calls"] = float(np.median([e[0].elapsed_time(e[4]) for e in evs]))
    roofline, breakdown, traced_ms = None, None, None
    if not args.no_trace:
        rx.rslx_trace_begin(1 << 17)
        t2 = time.perf_counter()
        for it in range(args.steps):
            step(args.warmup + args.steps + it, False)
        torch.cuda.synchronize()
        traced_ms = (time.perf_counter() - t2) * 1e3 / args.steps
        roofline, breakdown = summarize_trace(rx.rslx_trace_end(), w, args.steps)
    graph_ms = None
    if not args.no_graph:       # the same iteration on device-resident counters, recorded once and replayed
        ctr = rx.dev_counters(act_step=(args.warmup + 2 * args.steps) * T, call_index=args.warmup + 2 * args.steps,
                              adam_step=adam_step.value)

        def step_dc():
            for t in range(T):
                reset = dones[t - 1] if t > 0 else dones[T - 1]
                rx.rslx_act_recurrent_dc(ga, ma, gc, mc, obs[t], obs[t], N, h_a, h_c, reset, h0_a if t == 0 else None,
                                         h0_c if t == 0 else None, 20250910, ctr, None, actions[t], logp[t], values[t], mu[t],
                                         sigma[t], 0, aws)
            rx.rslx_act_recurrent(None, None, gc, mc, None, obs[T], N, None, h_c, dones[T - 1], None, None, 0, 0, None, None, None,
                                  last, None, None, rx.ACT_VALUES_ONLY, aws)
            rx.rslx_gae(rewards, values, last, dones, None, T, N, w.gamma, w.lam, 1, adv, ret, gws)
            rx.rslx_ppo_update_recurrent_dc(ga, ma, gc, mc, rollout, dones, h0_a, h0_c, rx.PpoCfg(**cfg_kw), ctr, stats, uws)

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step_dc()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t3) * 1e3 / args.steps
    assert torch.isfinite(ma.params).all() and torch.isfinite(ga.params).all() and torch.isfinite(stats).all()
    fwd = lambda dims: sum(2 * i * o for i, o in zip(dims[:-1], dims[1:]))
    gru_fwd = lambda D: 2 * (D + H) * G * H
    gru_bwd = lambda D: 2 * D * G * H + 2 * 2 * H * G * H
    per_sample = 3 * (fwd(w.dims_actor) + fwd(w.dims_critic)) + gru_fwd(w.Da) + gru_fwd(w.Dc) + gru_bwd(w.Da) + gru_bwd(w.Dc)
    act_flops = fwd(w.dims_actor) + fwd(w.dims_critic) + gru_fwd(w.Da) + gru_fwd(w.Dc)
    return {
        "metric": "recurrent PPO (%s memories, BPTT) transitions/sec: act + GAE + update, 1 GPU" % ("LSTM" if lstm else "GRU"),
        "value": round(B / (ms_per_step * 1e-3), 1),
        "unit": "transitions/s (whole iteration: %d act + GAE + %dx%d PPO update)" % (T, w.epochs, w.minibatches),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: N=%d envs, T=%d, obs %d, act %d, %s %d + MLP %s ELU per network, %d epochs x %d minibatches "
                               "of %d environment columns" % (w.name, N, T, w.Da, A, "LSTM" if lstm else "GRU", H, list(w.hidden),
                                                             w.epochs, w.minibatches, N // w.minibatches)},
        "phase_ms": {k: round(v, 4) for k, v in med.items()},
        "update_tflops": round(per_sample * B * w.epochs / (med["update"] * 1e-3) / 1e12, 2),
        "act_tflops": round(act_flops * (T + 1) * N / (med["act"] * 1e-3) / 1e12, 2),
        "act_env_steps_per_s": round(T * N / (med["act_calls"] * 1e-3), 1),
        "traced_ms_per_step": None if traced_ms is None else round(traced_ms, 4),
        "graph_replay": None if graph_ms is None else {"ms_per_step": round(graph_ms, 4),
                                                       "value": round(B / (graph_ms * 1e-3), 1)},
        "roofline": roofline, "kernels": breakdown,
    }


def summarize_trace(trace, w, steps):
    """Roofline of the dominant kernel and the per-kernel breakdown, from the library's own HIP-event trace."""
    kinds = {}
    for name, flops, nbytes, ms in trace:
        k = kinds.setdefault(name, dict(n=0, ms=0.0, flops=0.0, bytes=0.0))
        k["n"] += 1; k["ms"] += ms; k["flops"] += flops; k["bytes"] += nbytes
    dom = max(kinds, key=lambda k: kinds[k]["ms"])
    d = kinds[dom]
    achieved = d["flops"] / (d["ms"] * 1e-3) / 1e12
    roofline = dict(bound="mfma", kernel=dom, achieved=round(achieved, 2), peak=FP32_MFMA_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=round(achieved / FP32_MFMA_PEAK_TFLOPS, 4),
                    traffic=hbm_traffic_per_launch(w.name, dom),
                    traffic_source="profiles/%s_iteration_hbm_traffic.txt (rocprofv3 FETCH_SIZE / WRITE_SIZE of these kernel sources)" % w.name,
                    launches=d["n"], avg_launch_us=round(d["ms"] * 1e3 / d["n"], 2),
                    flops_per_launch=d["flops"] / d["n"])
    breakdown = {k: dict(launches=v["n"], total_ms_per_step=round(v["ms"] / steps, 4),
                         tflops=round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2) if v["flops"] else None,
                         gbs=round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["bytes"] else None)
                 for k, v in sorted(kinds.items(), key=lambda kv: -kv[1]["ms"])}

    return roofline, breakdown


def streaming_kernels(rx, torch, T, N, n_params):
    """HBM-bound pieces on their own: GAE (+ advantage normalisation) and clip + Adam, at the workload's size
    (a few MB: cache resident and launch-latency bound) and at a size that shows the achieved HBM bandwidth."""
    def timeit(f, reps):
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            f()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    out = {}
    for label, n_env in (("gae_on_config", N), ("gae_off_config_2^20_envs", 1 << 20)):
        r = torch.randn(T, n_env, device="cuda"); V = torch.randn(T, n_env, device="cuda"); Vl = torch.randn(n_env, device="cuda")
        d = (torch.rand(T, n_env, device="cuda") < 0.001).to(torch.uint8)
        adv = torch.empty(T, n_env, device="cuda"); ret = torch.empty(T, n_env, device="cuda")
        ws = rx.workspace(rx.rslx_gae_workspace_bytes(T, n_env))
        ms = timeit(lambda: rx.rslx_gae(r, V, Vl, d, None, T, n_env, 0.99, 0.95, 1, adv, ret, ws), 20)
        nbytes = 25.0 * T * n_env + 4.0 * n_env       # 17 B/element scan + 8 B/element normalisation pass
        out[label] = {"us": round(ms * 1e3, 2), "GB/s": round(nbytes / ms / 1e6, 1), "frac_of_hbm_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
        del r, V, Vl, d, adv, ret
    for label, n in (("adam_on_config", n_params), ("adam_off_config_64M_params", 1 << 26)):
        p = torch.randn(n, device="cuda"); g = torch.randn(n, device="cuda") * 0.01
        m = torch.zeros(n, device="cuda"); v = torch.zeros(n, device="cuda")
        ws = rx.workspace(rx.rslx_adam_workspace_bytes(n)); st = ctypes.c_int64(0)
        ms = timeit(lambda: rx.rslx_adam_step(p, g, m, v, n, 1e-3, 0.9, 0.999, 1e-8, 1.0, st, None, ws), 10)
        nbytes = 32.0 * n                               # 4 B/param squared-norm pass + 28 B/param clip + Adam
        out[label] = {"us": round(ms * 1e3, 2), "GB/s": round(nbytes / ms / 1e6, 1), "frac_of_hbm_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
        del p, g, m, v
    return out


def cpu_baseline(w, inp):
    """The fp64 numpy oracle on the host cores, as it stands.  All cores: the whole iteration (act loop, GAE and
    every update epoch) on the headline workload; on the larger workloads one update epoch is timed and scaled to
    the epoch count (said in `sample`).  One thread: two act steps and one optimiser step, scaled to the
    iteration (a bounded sample: the whole iteration takes minutes on one core)."""
    import numpy as np
    from oracle import ppo as oppo, gae as ogae, rng as orng
    from threadpoolctl import threadpool_info, threadpool_limits
    pools = [p for p in threadpool_info() if p.get("user_api") == "blas"] or threadpool_info()
    cores = max([p.get("num_threads", 1) for p in pools] or [os.cpu_count()])
    blas = ", ".join(sorted({"%s %s" % (p.get("internal_api", "?"), p.get("version", "")) for p in pools})) or "unknown BLAS"
    T, N, A, B = w.T, w.N, w.A, w.B
    act_step = lambda t: oppo.act(inp["actor"], inp["critic"], w.dims_actor, w.dims_critic, inp["obs"][t], inp["obs"][t],
                                  orng.act_noise(1, t, N, A))
    t0 = time.perf_counter()
    outs = [act_step(t) for t in range(T)]
    lastv = oppo.act(inp["actor"], inp["critic"], w.dims_actor, w.dims_critic, inp["obs"][T], inp["obs"][T], np.zeros((N, A)))["values"]
    t_act = time.perf_counter() - t0
    vals = np.stack([o["values"] for o in outs])
    t0 = time.perf_counter()
    adv, ret = ogae.gae(inp["rewards"], vals, lastv, inp["dones"], w.gamma, w.lam, timeouts=inp.get("timeouts"))
    advn = ogae.normalize_advantages(adv)
    t_gae = time.perf_counter() - t0
    stack = lambda k: np.stack([o[k] for o in outs])
    flat = dict(obs_a=inp["obs"][:T].reshape(B, -1), obs_c=inp["obs"][:T].reshape(B, -1), actions=stack("actions").reshape(B, A),
                logp=stack("logp").reshape(B), values=vals.reshape(B), mu=stack("mu").reshape(B, A),
                sigma=stack("sigma").reshape(B, A), adv=advn.reshape(B), returns=ret.reshape(B))
    whole = w.name == "flat" or B * w.epochs <= 500000          # the whole update fits the time budget
    epochs_timed = w.epochs if whole else 1
    cfg = oppo.PPOConfig(clip=w.clip, value_coef=w.value_coef, entropy_coef=w.entropy_coef, max_grad_norm=w.max_grad_norm,
                         lr=w.lr, epochs=epochs_timed, minibatches=w.minibatches, seed=1)
    na, nc = inp["actor"].size, inp["critic"].size
    opt0 = lambda: dict(m_a=np.zeros(na), v_a=np.zeros(na), m_c=np.zeros(nc), v_c=np.zeros(nc), step=0)
    sym = None
    if w.symmetry:
        sym = oppo.SymSpec(inp["perm_obs"], inp["sign_obs"], inp["perm_obs"], inp["sign_obs"], inp["perm_act"], inp["sign_act"], w.mirror_loss_coef)
    t0 = time.perf_counter()
    oppo.ppo_update(inp["actor"], inp["critic"], w.dims_actor, w.dims_critic, flat, cfg, opt0(), sym)
    t_upd = (time.perf_counter() - t0) * (w.epochs / epochs_timed)
    total = t_act + t_gae + t_upd
    # one thread, bounded sample
    mb = B // w.minibatches
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        for t in range(2):
            act_step(t)
        t1_act = (time.perf_counter() - t0) / 2 * (T + 1)
        t0 = time.perf_counter()
        oppo.ppo_update(inp["actor"], inp["critic"], w.dims_actor, w.dims_critic, {k: v[:mb] for k, v in flat.items()},
                        oppo.PPOConfig(clip=cfg.clip, value_coef=cfg.value_coef, entropy_coef=cfg.entropy_coef,
                                       max_grad_norm=cfg.max_grad_norm, lr=cfg.lr, epochs=1, minibatches=1, seed=1), opt0(), sym)
        t1_upd = (time.perf_counter() - t0) * w.epochs * w.minibatches
    return {"value": round(B / total, 1), "unit": "transitions/s (whole iteration)", "cores": int(cores), "kind": "oracle",
            "sample": "fp64 numpy oracle (%s, %d threads): whole act loop (%.2f s), GAE (%.3f s) and %s (%.2f s) timed"
                      % (blas, cores, t_act, t_gae, "all %d update epochs" % w.epochs if whole
                         else "1 of %d update epochs, multiplied by %d" % (w.epochs, w.epochs), t_upd),
            "one_thread": {"value": round(B / (t1_act + t_gae + t1_upd), 1), "cores": 1,
                           "sample": "2 of %d act steps and 1 of %d optimiser steps timed on one thread and scaled to the iteration "
                                     "(%.1f s + %.1f s)" % (T + 1, w.epochs * w.minibatches, t1_act, t1_upd)}}


if __name__ == "__main__":
    main()
