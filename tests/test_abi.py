"""Host-side checks of the C ABI that need no GPU: every declared symbol is exported, and invalid
arguments are rejected with an error code before anything is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest
import torch

import paper_2509_10771_amd as rx
from paper_2509_10771_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "rslx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(rslx_[a-z_0-9]+)\s*\(", text)))
    assert declared == sorted(B.EXPORTS)
    for name in declared:
        assert hasattr(rx.lib, name), name
    assert rx.rslx_version() == 100


def test_binding_signatures_have_the_declared_arity():
    """Every prototype in the header and its ctypes signature in the binding take the same number of arguments."""
    text = open(os.path.join(ROOT, "include", "rslx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    protos = re.findall(r"\b(rslx_[a-z_0-9]+)\s*\(([^()]*)\)\s*;", text)
    assert len(protos) == len(B.EXPORTS)
    for name, args in protos:
        n = 0 if args.strip() in ("", "void") else len(args.split(","))
        fn = getattr(rx.lib, name)
        assert fn.argtypes is not None and len(fn.argtypes) == n, (name, n, fn.argtypes)


def test_recurrent_argument_errors():
    mlp_a, mlp_c = _cpu_mlp((8, 8, 2), True), _cpu_mlp((8, 8, 1))
    gru = rx.Gru(4, 8, torch.zeros(3 * 8 * (4 + 8 + 2)), trainable=True)
    lstm = rx.Lstm(4, 8, torch.zeros(4 * 8 * (4 + 8 + 2)), trainable=True)
    assert (gru.state_width, lstm.state_width) == (8, 16)
    z = lambda *s: torch.zeros(*s)
    ro = rx.Rollout(3, 4, z(12, 4), z(12, 4), z(12, 2), z(12), z(12), z(12, 2), z(12, 2), z(12), z(12))
    assert rx.rslx_ppo_update_recurrent_workspace_bytes(gru, mlp_a, gru, mlp_c, ro, rx.PpoCfg(minibatches=2)) > 0
    assert rx.rslx_ppo_update_recurrent_workspace_bytes(lstm, mlp_a, lstm, mlp_c, ro, rx.PpoCfg(minibatches=2)) > 0
    with pytest.raises(rx.RslxError, match="different cells"):
        rx.rslx_ppo_update_recurrent_workspace_bytes(gru, mlp_a, lstm, mlp_c, ro, rx.PpoCfg(minibatches=2))
    with pytest.raises(rx.RslxError, match="multiple of minibatches"):
        rx.rslx_ppo_update_recurrent_workspace_bytes(gru, mlp_a, gru, mlp_c, ro, rx.PpoCfg(minibatches=3))
    bad = rx.Memory(7, 4, 8, torch.zeros(3 * 8 * (4 + 8 + 2)), trainable=True)
    with pytest.raises(rx.RslxError, match="unknown cell"):
        rx.rslx_ppo_update_recurrent_workspace_bytes(bad, mlp_a, bad, mlp_c, ro, rx.PpoCfg(minibatches=2))
    with pytest.raises(rx.RslxError, match="memory width"):
        rx.rslx_bc_update_recurrent_workspace_bytes(gru, _cpu_mlp((6, 8, 2)), 3, 4, rx.BcCfg(minibatches=2))


def _cpu_mlp(dims, log_std=False, trainable=True):
    n = sum(i * o + o for i, o in zip(dims[:-1], dims[1:])) + (dims[-1] if log_std else 0)
    return rx.Mlp(dims, torch.zeros(n), trainable=trainable, has_log_std=log_std)


def test_gae_and_perm_argument_errors():
    assert rx.lib.rslx_gae(None, None, None, None, None, 3, 4, 0.9, 0.9, 1, None, None, None, 0, None) == 1
    assert b"null" in rx.lib.rslx_last_error()
    assert rx.lib.rslx_gae(None, None, None, None, None, -1, 4, 0.9, 0.9, 1, None, None, None, 0, None) == 2
    assert rx.lib.rslx_gae(None, None, None, None, None, 0, 4, 0.9, 0.9, 1, None, None, None, 0, None) == 0   # empty: no-op
    assert rx.lib.rslx_permutation(1, 2, 0, 0, None, None, 0, None) == 0
    assert rx.lib.rslx_permutation(1, 2, 0, 10, None, None, 0, None) == 1
    assert rx.rslx_permutation_workspace_bytes(100000) > 100000 * 12


def test_ppo_update_argument_errors():
    actor, critic = _cpu_mlp((4, 8, 2), True), _cpu_mlp((4, 8, 1))
    T, N = 3, 5
    z = lambda *s: torch.zeros(*s)
    ro = rx.Rollout(T, N, z(15, 4), z(15, 4), z(15, 2), z(15), z(15), z(15, 2), z(15, 2), z(15), z(15))
    with pytest.raises(rx.RslxError, match="multiple of minibatches"):
        rx.rslx_ppo_update_workspace_bytes(actor, critic, ro, rx.PpoCfg(minibatches=4))
    n = rx.rslx_ppo_update_workspace_bytes(actor, critic, ro, rx.PpoCfg(minibatches=3))
    assert n > 0
    step = C.c_int64(0)
    with pytest.raises(rx.RslxError, match="workspace"):
        rx.rslx_ppo_update(actor, critic, ro, rx.PpoCfg(minibatches=3), None, None, step, z(15, 8), torch.zeros(16, dtype=torch.uint8))
    assert step.value == 0
    bad = rx.Sym([1, 2, 0, 3], [1, 1, 1, 1], [0, 1, 2, 3], [1, 1, 1, 1], [1, 0], [1, -1], device=None)
    with pytest.raises(rx.RslxError, match="involutive"):
        rx.rslx_ppo_update_workspace_bytes(actor, critic, ro, rx.PpoCfg(minibatches=3), bad)
    wrong = _cpu_mlp((5, 8, 1))
    with pytest.raises(rx.RslxError, match="widths"):
        rx.rslx_ppo_update_workspace_bytes(actor, wrong, ro, rx.PpoCfg(minibatches=3))
    frozen = _cpu_mlp((4, 8, 1), trainable=False)
    with pytest.raises(rx.RslxError, match="required"):
        rx.rslx_ppo_update(actor, frozen, ro, rx.PpoCfg(minibatches=3), None, None, step, z(15, 8), torch.zeros(n, dtype=torch.uint8))


def test_bc_sym_rnd_argument_errors():
    student, teacher = _cpu_mlp((4, 8, 2)), _cpu_mlp((6, 8, 3), trainable=False)
    with pytest.raises(rx.RslxError, match="action widths"):
        rx.rslx_bc_update_workspace_bytes(student, teacher, 16, rx.BcCfg(minibatches=4))
    with pytest.raises(rx.RslxError, match="multiple"):
        rx.rslx_bc_update_workspace_bytes(student, None, 15, rx.BcCfg(minibatches=4))
    bad = rx.Sym([1, 0], [1, -1], [0, 1], [1, 1], [0, 1], [1, 1], device=None)
    x = torch.zeros(3, 2)
    with pytest.raises(rx.RslxError, match="involutive"):
        rx.rslx_sym_augment(bad, x, None, 3, 2, 2, torch.zeros(6, 2), None)
    t, p = _cpu_mlp((4, 8, 3), trainable=False), _cpu_mlp((4, 8, 2), trainable=False)
    with pytest.raises(rx.RslxError, match="shape"):
        rx.rslx_rnd(t, p, torch.zeros(5, 4), 5, 4, None, 4, torch.zeros(3), 0.5, 1, torch.zeros(5), None, torch.zeros(1 << 16, dtype=torch.uint8))
