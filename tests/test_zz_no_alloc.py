"""The entry point that allocates nothing (rslx_gae_noalloc) against rslx_gae: same kernels on a scratch array
inside the library's device image, so the outputs must agree bit for bit; two calls in a row, the second on a
smaller input (the array keeps the first call's contents).  Also checked against the oracle to the GAE bound."""
import numpy as np
import pytest
import torch

from oracle import gae as ogae
from gpu_util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rx():
    import paper_2509_10771_amd as m
    m.rslx_device_check()
    return m


def _inputs(T, N, seed):
    g = np.random.default_rng(seed)
    return dict(rewards=g.normal(0.5, 0.3, (T, N)).astype(np.float32), values=g.normal(0, 1, (T, N)).astype(np.float32),
                last=g.normal(0, 1, N).astype(np.float32), dones=(g.random((T, N)) < 0.02).astype(np.uint8),
                timeouts=(g.random((T, N)) < 0.01).astype(np.uint8))


def _both(rx, T, N, seed, normalize, with_timeouts):
    i = _inputs(T, N, seed)
    if with_timeouts:
        i["dones"] |= i["timeouts"]
    d = {k: dev(v) for k, v in i.items()}
    to = d["timeouts"] if with_timeouts else None
    adv0, ret0, adv1, ret1 = (torch.full((T, N), float("nan"), device="cuda") for _ in range(4))
    ws = rx.workspace(rx.rslx_gae_workspace_bytes(T, N))
    rx.rslx_gae(d["rewards"], d["values"], d["last"], d["dones"], to, T, N, 0.99, 0.95, normalize, adv0, ret0, ws)
    rx.rslx_gae_noalloc(d["rewards"], d["values"], d["last"], d["dones"], to, T, N, 0.99, 0.95, normalize, adv1, ret1)
    torch.cuda.synchronize()
    assert torch.equal(adv0, adv1) and torch.equal(ret0, ret1), (T, N, normalize)
    a_ref, r_ref = ogae.gae(i["rewards"], i["values"], i["last"], i["dones"], 0.99, 0.95, timeouts=i["timeouts"] if with_timeouts else None)
    if normalize:
        a_ref = ogae.normalize_advantages(a_ref)
    assert np.max(np.abs(host(ret1) - r_ref)) <= 1e-5 * max(1.0, np.max(np.abs(r_ref)))
    assert np.max(np.abs(host(adv1) - a_ref)) <= 2e-5 * max(1.0, np.max(np.abs(a_ref)))


def test_noalloc_gae_matches_rslx_gae_on_consecutive_calls(rx):
    _both(rx, 24, 70001, 1, True, True)      # 274 workgroups of 256 lanes, ragged tail
    _both(rx, 24, 4096, 2, True, False)      # smaller: 64 workgroups of 64 lanes read fewer partial sums than the last call left
    _both(rx, 7, 300, 3, True, True)
    _both(rx, 24, 4096, 4, False, False)     # without normalisation the scratch is not touched
    _both(rx, 1, 3, 5, True, False)


def test_noalloc_gae_limits_and_errors(rx):
    N = rx.GAE_NOALLOC_MAX_ENVS + 1
    z = torch.zeros(8, device="cuda")
    with pytest.raises(rx.RslxError, match="exceeds the built-in scratch"):
        rx.rslx_gae_noalloc(z, z, z, z.to(torch.uint8), None, 1, N, 0.99, 0.95, 1, z, z)
    with pytest.raises(rx.RslxError, match="null pointer"):
        rx.rslx_gae_noalloc(None, z, z, z.to(torch.uint8), None, 1, 8, 0.99, 0.95, 1, z, z)
    rx.rslx_gae_noalloc(None, None, None, None, None, 0, 8, 0.99, 0.95, 1, None, None)     # empty roll-out: no-op


def test_noalloc_gae_at_its_size_limit(rx):
    N = rx.GAE_NOALLOC_MAX_ENVS
    _both(rx, 2, N, 6, True, False)
