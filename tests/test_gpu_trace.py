"""The launch trace (measurement aid): one record per launch with its own pair of events, launches beyond the
record limit are counted and reported instead of stretching the last record, and an update call with nothing to do
launches nothing and changes nothing."""
import ctypes as C

import numpy as np
import pytest
import torch

from workloads import WORKLOADS
from gpu_util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rx():
    import paper_2509_10771_amd as m
    m.rslx_device_check()
    return m


def _gae_call(rx, T=4, N=256):
    g = np.random.default_rng(0)
    r, v = dev(g.normal(size=(T, N)).astype(np.float32)), dev(g.normal(size=(T, N)).astype(np.float32))
    last, d = dev(g.normal(size=N).astype(np.float32)), dev(np.zeros((T, N), np.uint8))
    adv, ret = torch.empty(T, N, device="cuda"), torch.empty(T, N, device="cuda")
    ws = rx.workspace(rx.rslx_gae_workspace_bytes(T, N))
    return lambda: rx.rslx_gae(r, v, last, d, None, T, N, 0.99, 0.95, 0, adv, ret, ws)


def test_trace_records_one_entry_per_launch(rx):
    call = _gae_call(rx)
    call(); torch.cuda.synchronize()
    rx.rslx_trace_begin(64)
    for _ in range(5):
        call()
    torch.cuda.synchronize()
    rec = rx.rslx_trace_end()
    assert len(rec) == 5 and all(name == "gae_scan" for name, _, _, _ in rec)
    ms = np.array([m for _, _, _, m in rec])
    # every record spans its own launch: microseconds, and no record swallows the launches after it
    assert np.all(ms > 0) and np.all(ms < 1.0) and ms.max() < 20 * np.median(ms)


def test_trace_reports_launches_it_could_not_record(rx):
    call = _gae_call(rx)
    rx.rslx_trace_begin(2)
    for _ in range(6):
        call()
    torch.cuda.synchronize()
    with pytest.raises(rx.RslxError, match="4 launches were not recorded"):
        rx.rslx_trace_end()
    # the trace is usable again afterwards
    rx.rslx_trace_begin(8)
    call()
    torch.cuda.synchronize()
    assert len(rx.rslx_trace_end()) == 1


def test_update_with_zero_epochs_is_a_no_op(rx):
    import test_gpu_update as tu
    case = tu.Case(WORKLOADS["tiny"], 1)
    a, c, rnd = tu._nets(rx, case, case.actor0, case.critic0)
    ro, cfg = case.gpu_rollout(rx), case.gpu_cfg(rx, 0, case.w.minibatches)
    stats = torch.full((1, rx.NSTATS), 7.0, device="cuda")
    before = (a.params.clone(), c.params.clone())
    step = C.c_int64(11)
    ws = rx.workspace(max(rx.rslx_ppo_update_workspace_bytes(a, c, ro, cfg), 256))
    rx.rslx_trace_begin(16)
    rx.rslx_ppo_update(a, c, ro, cfg, None, rnd, step, stats, ws)
    torch.cuda.synchronize()
    rec = rx.rslx_trace_end()
    assert step.value == 11 and torch.equal(a.params, before[0]) and torch.equal(c.params, before[1])
    assert torch.all(stats == 7.0)
    assert all(name == "stage_input" for name, _, _, _ in rec), rec
