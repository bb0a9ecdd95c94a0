"""The largest sizes the entry points are run at anywhere in this repository (the off-configuration sizes of the
bandwidth figures, a batch far beyond the layer-fused inference launch, a permutation of 2^24 rows), each compared with
the fp64 oracle in full: the oracle's steps are vectorised over the batch, so whole-array comparisons still take seconds."""
import ctypes as C
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import rng as orng, adam as oadam, ppo as oppo
from workloads import WORKLOADS, make_inputs
from gpu_util import dev, host, f32
import test_gpu_basic as B

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rx():
    import paper_2509_10771_amd as m
    m.rslx_device_check()
    return m


def test_gae_at_a_million_environments(rx):
    B._gae_case(rx, 24, 1 << 20, 0.99, 0.95, 0.02, True, False, seed=3)
    B._gae_case(rx, 24, (1 << 20) - 3, 0.99, 0.95, 0.02, False, True, seed=4)      # normalised, ragged last block


def test_permutation_of_sixteen_million_rows(rx):
    n = 1 << 24
    ws = rx.workspace(rx.rslx_permutation_workspace_bytes(n))
    out = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    rx.rslx_permutation(7, 3, 2, n, out, ws)
    torch.cuda.synchronize()
    assert np.array_equal(host(out), orng.permutation(7, 3, 2, n))


def test_adam_on_sixty_four_million_parameters(rx):
    n = 1 << 26
    g = np.random.default_rng(26)
    th = g.standard_normal(n, dtype=np.float32)
    gr = g.standard_normal(n, dtype=np.float32) * np.float32(1e-4)
    p, gg, m, v = dev(th), dev(gr), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    step = C.c_int64(0)
    norm_out = torch.zeros(1, device="cuda")
    ws = rx.workspace(rx.rslx_adam_workspace_bytes(n))
    rx.rslx_adam_step(p, gg, m, v, n, 1e-3, 0.9, 0.999, 1e-8, 0.5, step, norm_out, ws)
    torch.cuda.synchronize()
    norm = oadam.global_norm([gr])
    assert abs(host(norm_out)[0] - norm) <= 1e-5 * norm
    scale = oadam.clip_scale(norm, 0.5)
    assert scale < 1.0
    th1, m1, v1, _ = oadam.adam_step(th.astype(np.float64), scale * gr.astype(np.float64), np.zeros(n), np.zeros(n), 0,
                                     f32(1e-3), f32(0.9), f32(0.999), f32(1e-8))
    np.testing.assert_allclose(host(p), th1, rtol=2e-6, atol=2e-7)
    np.testing.assert_allclose(host(m), m1, rtol=1e-5, atol=1e-10)
    np.testing.assert_allclose(host(v), v1, rtol=1e-5, atol=1e-14)


def test_act_on_131072_rows(rx):
    w = replace(WORKLOADS["flat"].scaled(131072), T=1)
    inp = make_inputs(w)
    inp["actor"][-w.A:] = np.random.default_rng(5).normal(scale=0.3, size=w.A).astype(np.float32)
    B._act_case(rx, w, inp, 131072, use_eps=False)
