"""ctypes binding with the same names as the C ABI in include/rslx.h (argument marshalling only)."""
import ctypes as C
import os

import torch

__all__ = [
    "RslxError", "lib", "Mlp", "Rollout", "PpoCfg", "BcCfg", "Sym", "RndTrain", "workspace", "NSTATS",
    "rslx_version", "rslx_device_check", "rslx_permutation", "rslx_permutation_workspace_bytes",
    "rslx_act", "rslx_act_workspace_bytes", "rslx_gae", "rslx_gae_workspace_bytes",
    "rslx_adam_step", "rslx_adam_workspace_bytes", "rslx_ppo_update", "rslx_ppo_update_workspace_bytes",
    "rslx_bc_update", "rslx_bc_update_workspace_bytes", "rslx_sym_augment", "rslx_rnd", "rslx_rnd_workspace_bytes",
    "ACT_DETERMINISTIC", "ACT_VALUES_ONLY", "EXPORTS", "rslx_trace_begin", "rslx_trace_end",
    "dev_counters", "rslx_act_dc", "rslx_ppo_update_dc", "rslx_bc_update_dc", "rslx_bc_collect_workspace_bytes",
    "rslx_bc_collect", "Memory", "Gru", "Lstm", "CELL_GRU", "CELL_LSTM", "rslx_act_recurrent_workspace_bytes", "rslx_act_recurrent",
    "rslx_ppo_update_recurrent_workspace_bytes", "rslx_ppo_update_recurrent", "rslx_memory_step_workspace_bytes",
    "rslx_memory_step", "rslx_bc_update_recurrent_workspace_bytes", "rslx_bc_update_recurrent",
    "rslx_act_recurrent_dc", "rslx_ppo_update_recurrent_dc", "rslx_gae_noalloc", "GAE_NOALLOC_MAX_ENVS",
]

MAX_LAYERS = 8
NSTATS = 8
ACT_DETERMINISTIC = 1
ACT_VALUES_ONLY = 2

EXPORTS = [
    "rslx_version", "rslx_last_error", "rslx_device_check", "rslx_permutation_workspace_bytes", "rslx_permutation",
    "rslx_act_workspace_bytes", "rslx_act", "rslx_gae_workspace_bytes", "rslx_gae", "rslx_adam_workspace_bytes",
    "rslx_adam_step", "rslx_ppo_update_workspace_bytes", "rslx_ppo_update", "rslx_bc_update_workspace_bytes",
    "rslx_bc_update", "rslx_sym_augment", "rslx_rnd_workspace_bytes", "rslx_rnd", "rslx_trace_begin", "rslx_trace_end",
    "rslx_act_dc", "rslx_ppo_update_dc", "rslx_bc_update_dc", "rslx_bc_collect_workspace_bytes", "rslx_bc_collect",
    "rslx_act_recurrent_workspace_bytes", "rslx_act_recurrent", "rslx_ppo_update_recurrent_workspace_bytes",
    "rslx_ppo_update_recurrent", "rslx_memory_step_workspace_bytes", "rslx_memory_step",
    "rslx_bc_update_recurrent_workspace_bytes", "rslx_bc_update_recurrent", "rslx_act_recurrent_dc",
    "rslx_ppo_update_recurrent_dc", "rslx_gae_noalloc",
]
GAE_NOALLOC_MAX_ENVS = 1 << 20

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "librslx.so")


class RslxError(RuntimeError):
    pass


if not os.path.exists(_LIB_PATH):
    raise ImportError("librslx.so is missing at %s: build it with `python paper_2509_10771_amd/build.py`; "
                      "there is no fallback path" % _LIB_PATH)
lib = C.CDLL(_LIB_PATH)

_fp = C.POINTER(C.c_float)
_vp = C.c_void_p


class _CMlp(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("dims", C.c_int32 * (MAX_LAYERS + 1)), ("elu_alpha", C.c_float),
                ("has_log_std", C.c_int32), ("params", _vp), ("grads", _vp), ("adam_m", _vp), ("adam_v", _vp)]


class _CMemory(C.Structure):
    _fields_ = [("cell", C.c_int32), ("in_dim", C.c_int32), ("hidden", C.c_int32), ("params", _vp), ("grads", _vp),
                ("adam_m", _vp), ("adam_v", _vp)]


class _CRollout(C.Structure):
    _fields_ = [("T", C.c_int32), ("N", C.c_int32), ("Da", C.c_int32), ("Dc", C.c_int32), ("A", C.c_int32),
                ("obs_actor", _vp), ("obs_critic", _vp), ("actions", _vp), ("logp", _vp), ("values", _vp),
                ("mu", _vp), ("sigma", _vp), ("advantages", _vp), ("returns", _vp)]


class _CPpoCfg(C.Structure):
    _fields_ = [("clip", C.c_float), ("value_coef", C.c_float), ("entropy_coef", C.c_float), ("max_grad_norm", C.c_float),
                ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("adam_eps", C.c_float),
                ("epochs", C.c_int32), ("minibatches", C.c_int32), ("use_clipped_value_loss", C.c_int32),
                ("seed", C.c_uint64), ("call_index", C.c_uint64), ("epoch_offset", C.c_int32)]


class _CSym(C.Structure):
    _fields_ = [("perm_obs_a_host", _vp), ("sign_obs_a_host", _vp), ("perm_obs_c_host", _vp), ("sign_obs_c_host", _vp),
                ("perm_act_host", _vp), ("sign_act_host", _vp),
                ("perm_obs_a", _vp), ("sign_obs_a", _vp), ("perm_obs_c", _vp), ("sign_obs_c", _vp),
                ("perm_act", _vp), ("sign_act", _vp), ("mirror_loss_coef", C.c_float)]


class _CRndTrain(C.Structure):
    _fields_ = [("target", C.POINTER(_CMlp)), ("predictor", C.POINTER(_CMlp)), ("subset_idx", _vp),
                ("n_subset", C.c_int32), ("lr", C.c_float), ("adam_step", C.POINTER(C.c_int64))]


class _CBcCfg(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("adam_eps", C.c_float),
                ("max_grad_norm", C.c_float), ("epochs", C.c_int32), ("minibatches", C.c_int32),
                ("seed", C.c_uint64), ("call_index", C.c_uint64), ("epoch_offset", C.c_int32)]


class _CTraceRecord(C.Structure):
    _fields_ = [("kernel", C.c_char * 48), ("flops", C.c_double), ("bytes", C.c_double), ("ms", C.c_float)]


def _sig(name, restype, argtypes):
    f = getattr(lib, name)
    f.restype = restype
    f.argtypes = argtypes
    return f


_P = C.POINTER
_sig("rslx_version", C.c_int32, [])
_sig("rslx_last_error", C.c_char_p, [])
_sig("rslx_device_check", C.c_int32, [])
_sig("rslx_permutation_workspace_bytes", C.c_size_t, [C.c_int32])
_sig("rslx_permutation", C.c_int32, [C.c_uint64, C.c_uint64, C.c_int32, C.c_int32, _vp, _vp, C.c_size_t, _vp])
_sig("rslx_act_workspace_bytes", C.c_size_t, [_P(_CMlp), _P(_CMlp), C.c_int32])
_sig("rslx_act", C.c_int32, [_P(_CMlp), _P(_CMlp), _vp, _vp, C.c_int32, C.c_uint64, C.c_uint64, _vp, _vp, _vp, _vp, _vp,
                             _vp, C.c_uint32, _vp, C.c_size_t, _vp])
_sig("rslx_act_dc", C.c_int32, [_P(_CMlp), _P(_CMlp), _vp, _vp, C.c_int32, C.c_uint64, _vp, _vp, _vp, _vp, _vp, _vp,
                                _vp, C.c_uint32, _vp, C.c_size_t, _vp])
_sig("rslx_gae_workspace_bytes", C.c_size_t, [C.c_int32, C.c_int32])
_sig("rslx_gae", C.c_int32, [_vp, _vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_float, C.c_float, C.c_int32, _vp, _vp,
                             _vp, C.c_size_t, _vp])
_sig("rslx_gae_noalloc", C.c_int32, [_vp, _vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_float, C.c_float, C.c_int32, _vp, _vp, _vp])
_sig("rslx_adam_workspace_bytes", C.c_size_t, [C.c_int64])
_sig("rslx_adam_step", C.c_int32, [_vp, _vp, _vp, _vp, C.c_int64, C.c_float, C.c_float, C.c_float, C.c_float, C.c_float,
                                   _P(C.c_int64), _vp, _vp, C.c_size_t, _vp])
_sig("rslx_ppo_update_workspace_bytes", C.c_size_t, [_P(_CMlp), _P(_CMlp), _P(_CRollout), _P(_CPpoCfg), _P(_CSym), _P(_CRndTrain)])
_sig("rslx_ppo_update", C.c_int32, [_P(_CMlp), _P(_CMlp), _P(_CRollout), _P(_CPpoCfg), _P(_CSym), _P(_CRndTrain),
                                    _P(C.c_int64), _vp, _vp, C.c_size_t, _vp])
_sig("rslx_ppo_update_dc", C.c_int32, [_P(_CMlp), _P(_CMlp), _P(_CRollout), _P(_CPpoCfg), _P(_CSym), _P(_CRndTrain),
                                       _vp, _vp, _vp, C.c_size_t, _vp])
_sig("rslx_bc_update_workspace_bytes", C.c_size_t, [_P(_CMlp), _P(_CMlp), C.c_int32, _P(_CBcCfg)])
_sig("rslx_bc_update", C.c_int32, [_P(_CMlp), _P(_CMlp), _vp, _vp, _vp, C.c_int32, _P(_CBcCfg), _P(C.c_int64), _vp, _vp,
                                   C.c_size_t, _vp])
_sig("rslx_bc_update_dc", C.c_int32, [_P(_CMlp), _P(_CMlp), _vp, _vp, _vp, C.c_int32, _P(_CBcCfg), _vp, _vp, _vp,
                                      C.c_size_t, _vp])
_sig("rslx_bc_collect_workspace_bytes", C.c_size_t, [_P(_CMlp), _P(_CMlp), C.c_int32])
_sig("rslx_bc_collect", C.c_int32, [_P(_CMlp), _P(_CMlp), _vp, _vp, C.c_int32, _vp, _vp, _vp, C.c_size_t, _vp])
_sig("rslx_act_recurrent_workspace_bytes", C.c_size_t, [_P(_CMemory), _P(_CMlp), _P(_CMemory), _P(_CMlp), C.c_int32])
_sig("rslx_act_recurrent", C.c_int32, [_P(_CMemory), _P(_CMlp), _P(_CMemory), _P(_CMlp), _vp, _vp, C.c_int32, _vp, _vp, _vp, _vp,
                                       _vp, C.c_uint64, C.c_uint64, _vp, _vp, _vp, _vp, _vp, _vp, C.c_uint32, _vp,
                                       C.c_size_t, _vp])
_sig("rslx_act_recurrent_dc", C.c_int32, [_P(_CMemory), _P(_CMlp), _P(_CMemory), _P(_CMlp), _vp, _vp, C.c_int32, _vp, _vp, _vp,
                                          _vp, _vp, C.c_uint64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, C.c_uint32, _vp,
                                          C.c_size_t, _vp])
_sig("rslx_ppo_update_recurrent_dc", C.c_int32, [_P(_CMemory), _P(_CMlp), _P(_CMemory), _P(_CMlp), _P(_CRollout), _vp, _vp, _vp,
                                                 _P(_CPpoCfg), _vp, _vp, _vp, C.c_size_t, _vp])
_sig("rslx_ppo_update_recurrent_workspace_bytes", C.c_size_t, [_P(_CMemory), _P(_CMlp), _P(_CMemory), _P(_CMlp), _P(_CRollout),
                                                               _P(_CPpoCfg)])
_sig("rslx_ppo_update_recurrent", C.c_int32, [_P(_CMemory), _P(_CMlp), _P(_CMemory), _P(_CMlp), _P(_CRollout), _vp, _vp, _vp,
                                              _P(_CPpoCfg), _P(C.c_int64), _vp, _vp, C.c_size_t, _vp])
_sig("rslx_memory_step_workspace_bytes", C.c_size_t, [_P(_CMemory), C.c_int32])
_sig("rslx_memory_step", C.c_int32, [_P(_CMemory), _vp, C.c_int32, _vp, _vp, _vp, _vp, _vp, C.c_size_t, _vp])
_sig("rslx_bc_update_recurrent_workspace_bytes", C.c_size_t, [_P(_CMemory), _P(_CMlp), C.c_int32, C.c_int32, _P(_CBcCfg)])
_sig("rslx_bc_update_recurrent", C.c_int32, [_P(_CMemory), _P(_CMlp), _vp, _vp, _vp, _vp, C.c_int32, C.c_int32, _P(_CBcCfg),
                                             _P(C.c_int64), _vp, _vp, C.c_size_t, _vp])
_sig("rslx_sym_augment", C.c_int32, [_P(_CSym), _vp, _vp, C.c_int32, C.c_int32, C.c_int32, _vp, _vp, _vp])
_sig("rslx_rnd_workspace_bytes", C.c_size_t, [_P(_CMlp), C.c_int32])
_sig("rslx_rnd", C.c_int32, [_P(_CMlp), _P(_CMlp), _vp, C.c_int32, C.c_int32, _vp, C.c_int32, _vp, C.c_float, C.c_int32,
                             _vp, _vp, _vp, C.c_size_t, _vp])


_sig("rslx_trace_begin", C.c_int32, [C.c_int32])
_sig("rslx_trace_end", C.c_int32, [_P(_CTraceRecord), C.c_int32, _P(C.c_int32)])


def _check(rc, what):
    if rc != 0:
        raise RslxError("%s failed with status %d: %s" % (what, rc, lib.rslx_last_error().decode()))


def _ptr(t):
    """Device (or host) address of a contiguous tensor; None -> NULL."""
    if t is None:
        return None
    assert t.is_contiguous(), "rslx needs contiguous tensors"
    return t.data_ptr()


def _stream():
    """torch's current stream; without a GPU (host-side argument checks only) the NULL stream."""
    return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None


def workspace(nbytes, device="cuda"):
    """Device scratch buffer for the *_workspace_bytes() queries."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


class Mlp:
    """A network over flat device tensors (layout in include/rslx.h)."""

    def __init__(self, dims, params, trainable=False, has_log_std=False, elu_alpha=1.0):
        self.dims = tuple(int(d) for d in dims)
        self.has_log_std = bool(has_log_std)
        n = sum(i * o + o for i, o in zip(self.dims[:-1], self.dims[1:])) + (self.dims[-1] if has_log_std else 0)
        assert params.dtype == torch.float32 and params.numel() == n, (params.numel(), n)
        self.params = params
        self.grads = torch.zeros_like(params) if trainable else None
        self.adam_m = torch.zeros_like(params) if trainable else None
        self.adam_v = torch.zeros_like(params) if trainable else None
        self.elu_alpha = float(elu_alpha)

    @property
    def c(self):
        s = _CMlp()
        s.n_layers = len(self.dims) - 1
        for i, d in enumerate(self.dims):
            s.dims[i] = d
        s.elu_alpha = self.elu_alpha
        s.has_log_std = int(self.has_log_std)
        s.params = _ptr(self.params)
        s.grads = _ptr(self.grads)
        s.adam_m = _ptr(self.adam_m)
        s.adam_v = _ptr(self.adam_v)
        return s


CELL_GRU, CELL_LSTM = 0, 1


class Memory:
    """Recurrent memory over a flat device buffer: W_ih [in, G H], b_ih [G H], W_hh [H, G H], b_hh [G H]
    (GRU: G = 3, state width H; LSTM: G = 4, packed state [h | c] of width 2 H)."""

    def __init__(self, cell, in_dim, hidden, params, trainable=False):
        self.cell, self.in_dim, self.hidden = int(cell), int(in_dim), int(hidden)
        self.gates = 4 if self.cell == CELL_LSTM else 3
        self.state_width = 2 * self.hidden if self.cell == CELL_LSTM else self.hidden
        assert params.numel() == self.gates * self.hidden * (self.in_dim + self.hidden + 2)
        self.params = params
        self.grads = torch.zeros_like(params) if trainable else None
        self.adam_m = torch.zeros_like(params) if trainable else None
        self.adam_v = torch.zeros_like(params) if trainable else None

    @property
    def c(self):
        return _CMemory(self.cell, self.in_dim, self.hidden, _ptr(self.params), _ptr(self.grads), _ptr(self.adam_m),
                        _ptr(self.adam_v))


def Gru(in_dim, hidden, params, trainable=False):
    return Memory(CELL_GRU, in_dim, hidden, params, trainable)


def Lstm(in_dim, hidden, params, trainable=False):
    return Memory(CELL_LSTM, in_dim, hidden, params, trainable)


class Rollout:
    def __init__(self, T, N, obs_actor, obs_critic, actions, logp, values, mu, sigma, advantages, returns):
        self.T, self.N = int(T), int(N)
        self.t = dict(obs_actor=obs_actor, obs_critic=obs_critic, actions=actions, logp=logp, values=values, mu=mu,
                      sigma=sigma, advantages=advantages, returns=returns)
        B = self.T * self.N
        self.Da, self.Dc, self.A = obs_actor.numel() // B, obs_critic.numel() // B, actions.numel() // B

    @property
    def c(self):
        s = _CRollout(self.T, self.N, self.Da, self.Dc, self.A)
        for k, v in self.t.items():
            setattr(s, k, _ptr(v))
        return s


class PpoCfg:
    def __init__(self, clip=0.2, value_coef=1.0, entropy_coef=0.01, max_grad_norm=1.0, lr=1e-3, beta1=0.9, beta2=0.999,
                 adam_eps=1e-8, epochs=5, minibatches=4, use_clipped_value_loss=True, seed=0, call_index=0, epoch_offset=0):
        self.c = _CPpoCfg(clip, value_coef, entropy_coef, max_grad_norm, lr, beta1, beta2, adam_eps, epochs, minibatches,
                          int(use_clipped_value_loss), seed, call_index, epoch_offset)


class BcCfg:
    def __init__(self, lr=1e-3, beta1=0.9, beta2=0.999, adam_eps=1e-8, max_grad_norm=0.0, epochs=2, minibatches=4, seed=0,
                 call_index=0, epoch_offset=0):
        self.c = _CBcCfg(lr, beta1, beta2, adam_eps, max_grad_norm, epochs, minibatches, seed, call_index, epoch_offset)


class Sym:
    """Mirror maps: host copies (int32 / float32 CPU tensors) plus device copies (device=None: none; rslx_ppo_update
    then uploads the host copies itself)."""

    def __init__(self, perm_obs_a, sign_obs_a, perm_obs_c, sign_obs_c, perm_act, sign_act, mirror_loss_coef=1.0, device="cuda"):
        host = [torch.as_tensor(perm_obs_a, dtype=torch.int32).contiguous(), torch.as_tensor(sign_obs_a, dtype=torch.float32).contiguous(),
                torch.as_tensor(perm_obs_c, dtype=torch.int32).contiguous(), torch.as_tensor(sign_obs_c, dtype=torch.float32).contiguous(),
                torch.as_tensor(perm_act, dtype=torch.int32).contiguous(), torch.as_tensor(sign_act, dtype=torch.float32).contiguous()]
        self.host = host
        self.dev = [h.to(device) for h in host] if device is not None else [None] * 6
        self.mirror_loss_coef = float(mirror_loss_coef)

    @property
    def c(self):
        s = _CSym()
        names = ["perm_obs_a", "sign_obs_a", "perm_obs_c", "sign_obs_c", "perm_act", "sign_act"]
        for n, h, d in zip(names, self.host, self.dev):
            setattr(s, n + "_host", _ptr(h))
            setattr(s, n, _ptr(d))
        s.mirror_loss_coef = self.mirror_loss_coef
        return s


class RndTrain:
    def __init__(self, target, predictor, subset_idx=None, lr=1e-3, adam_step=0):
        self.target, self.predictor, self.subset_idx, self.lr = target, predictor, subset_idx, float(lr)
        self.step = C.c_int64(int(adam_step))

    def c(self):
        self._ct, self._cp = self.target.c, self.predictor.c
        s = _CRndTrain(C.pointer(self._ct), C.pointer(self._cp), _ptr(self.subset_idx),
                       self.target.dims[0], self.lr, C.pointer(self.step))
        return s


def _ref(x):
    return None if x is None else C.byref(x)


def rslx_version():
    return lib.rslx_version()


def rslx_device_check():
    _check(lib.rslx_device_check(), "rslx_device_check")


def rslx_permutation_workspace_bytes(B):
    return lib.rslx_permutation_workspace_bytes(B)


def rslx_permutation(seed, call_index, epoch, B, perm_out, ws):
    _check(lib.rslx_permutation(seed, call_index, epoch, B, _ptr(perm_out), _ptr(ws), ws.numel(), _stream()), "rslx_permutation")


def rslx_act_workspace_bytes(actor, critic, N):
    return lib.rslx_act_workspace_bytes(_ref(actor.c) if actor is not None else None, _ref(critic.c), N)


def rslx_act(actor, critic, obs_actor, obs_critic, N, seed, step, eps, actions, logp, values, mu, sigma, flags, ws):
    ca = actor.c if actor is not None else None
    cc = critic.c
    _check(lib.rslx_act(_ref(ca), _ref(cc), _ptr(obs_actor), _ptr(obs_critic), N, seed, step, _ptr(eps), _ptr(actions),
                        _ptr(logp), _ptr(values), _ptr(mu), _ptr(sigma), flags, _ptr(ws), ws.numel(), _stream()), "rslx_act")


def dev_counters(act_step=0, call_index=0, adam_step=0, rnd_adam_step=0, device="cuda"):
    """rslx_dev_counters in device memory: int64 tensor [act_step, call_index, adam_step, rnd_adam_step]."""
    return torch.tensor([act_step, call_index, adam_step, rnd_adam_step], dtype=torch.int64, device=device)


def rslx_act_dc(actor, critic, obs_actor, obs_critic, N, seed, counters, eps, actions, logp, values, mu, sigma, flags, ws):
    """counters: int64 device tensor of 4 (dev_counters())."""
    ca = actor.c if actor is not None else None
    cc = critic.c
    _check(lib.rslx_act_dc(_ref(ca), _ref(cc), _ptr(obs_actor), _ptr(obs_critic), N, seed, _ptr(counters), _ptr(eps),
                           _ptr(actions), _ptr(logp), _ptr(values), _ptr(mu), _ptr(sigma), flags, _ptr(ws), ws.numel(),
                           _stream()), "rslx_act_dc")


def rslx_gae_workspace_bytes(T, N):
    return lib.rslx_gae_workspace_bytes(T, N)


def rslx_gae(rewards, values, last_values, dones, timeouts, T, N, gamma, lam, normalize_adv, advantages, returns, ws):
    _check(lib.rslx_gae(_ptr(rewards), _ptr(values), _ptr(last_values), _ptr(dones), _ptr(timeouts), T, N, gamma, lam,
                        int(normalize_adv), _ptr(advantages), _ptr(returns), _ptr(ws), ws.numel() if ws is not None else 0,
                        _stream()), "rslx_gae")


def rslx_gae_noalloc(rewards, values, last_values, dones, timeouts, T, N, gamma, lam, normalize_adv, advantages, returns):
    _check(lib.rslx_gae_noalloc(_ptr(rewards), _ptr(values), _ptr(last_values), _ptr(dones), _ptr(timeouts), T, N, gamma, lam,
                                int(normalize_adv), _ptr(advantages), _ptr(returns), _stream()), "rslx_gae_noalloc")


def rslx_adam_workspace_bytes(n):
    return lib.rslx_adam_workspace_bytes(n)


def rslx_adam_step(params, grads, m, v, n, lr, beta1, beta2, eps, max_grad_norm, adam_step, grad_norm_out, ws):
    """adam_step: ctypes.c_int64, updated in place."""
    _check(lib.rslx_adam_step(_ptr(params), _ptr(grads), _ptr(m), _ptr(v), n, lr, beta1, beta2, eps, max_grad_norm,
                              C.byref(adam_step), _ptr(grad_norm_out), _ptr(ws), ws.numel(), _stream()), "rslx_adam_step")


def rslx_ppo_update_workspace_bytes(actor, critic, rollout, cfg, sym=None, rnd=None):
    ca, cc, cr = actor.c, critic.c, rollout.c
    cs = sym.c if sym is not None else None
    cn = rnd.c() if rnd is not None else None
    n = lib.rslx_ppo_update_workspace_bytes(_ref(ca), _ref(cc), _ref(cr), _ref(cfg.c), _ref(cs), _ref(cn))
    if n == 0:
        raise RslxError("rslx_ppo_update_workspace_bytes: %s" % lib.rslx_last_error().decode())
    return n


def rslx_ppo_update(actor, critic, rollout, cfg, sym, rnd, adam_step, stats, ws):
    """adam_step: ctypes.c_int64, updated in place."""
    ca, cc, cr = actor.c, critic.c, rollout.c
    cs = sym.c if sym is not None else None
    cn = rnd.c() if rnd is not None else None
    _check(lib.rslx_ppo_update(_ref(ca), _ref(cc), _ref(cr), _ref(cfg.c), _ref(cs), _ref(cn), C.byref(adam_step),
                               _ptr(stats), _ptr(ws), ws.numel() if ws is not None else 0, _stream()), "rslx_ppo_update")


def rslx_ppo_update_dc(actor, critic, rollout, cfg, sym, rnd, counters, stats, ws):
    """counters: int64 device tensor of 4 (dev_counters()), advanced by the call's own kernels."""
    ca, cc, cr = actor.c, critic.c, rollout.c
    cs = sym.c if sym is not None else None
    cn = rnd.c() if rnd is not None else None
    _check(lib.rslx_ppo_update_dc(_ref(ca), _ref(cc), _ref(cr), _ref(cfg.c), _ref(cs), _ref(cn), _ptr(counters),
                                  _ptr(stats), _ptr(ws), ws.numel() if ws is not None else 0, _stream()), "rslx_ppo_update_dc")


def rslx_bc_update_workspace_bytes(student, teacher, B, cfg):
    cs = student.c
    ct = teacher.c if teacher is not None else None
    n = lib.rslx_bc_update_workspace_bytes(_ref(cs), _ref(ct), B, _ref(cfg.c))
    if n == 0:
        raise RslxError("rslx_bc_update_workspace_bytes: %s" % lib.rslx_last_error().decode())
    return n


def rslx_bc_update(student, teacher, obs_student, obs_teacher, targets, B, cfg, adam_step, stats, ws):
    cs = student.c
    ct = teacher.c if teacher is not None else None
    _check(lib.rslx_bc_update(_ref(cs), _ref(ct), _ptr(obs_student), _ptr(obs_teacher), _ptr(targets), B, _ref(cfg.c),
                              C.byref(adam_step), _ptr(stats), _ptr(ws), ws.numel() if ws is not None else 0, _stream()),
           "rslx_bc_update")


def rslx_bc_update_dc(student, teacher, obs_student, obs_teacher, targets, B, cfg, counters, stats, ws):
    """counters: int64 device tensor of 4 (dev_counters()); call_index and adam_step are used."""
    cs = student.c
    ct = teacher.c if teacher is not None else None
    _check(lib.rslx_bc_update_dc(_ref(cs), _ref(ct), _ptr(obs_student), _ptr(obs_teacher), _ptr(targets), B, _ref(cfg.c),
                                 _ptr(counters), _ptr(stats), _ptr(ws), ws.numel() if ws is not None else 0, _stream()),
           "rslx_bc_update_dc")


def rslx_bc_collect_workspace_bytes(student, teacher, N):
    return lib.rslx_bc_collect_workspace_bytes(_ref(student.c), _ref(teacher.c), N)


def rslx_bc_collect(student, teacher, obs_student, obs_teacher, N, actions, targets, ws):
    cs = student.c if student is not None else None
    ct = teacher.c if teacher is not None else None
    _check(lib.rslx_bc_collect(_ref(cs), _ref(ct), _ptr(obs_student), _ptr(obs_teacher), N, _ptr(actions), _ptr(targets),
                               _ptr(ws), ws.numel() if ws is not None else 0, _stream()), "rslx_bc_collect")


def rslx_act_recurrent_workspace_bytes(gru_actor, actor, gru_critic, critic, N):
    ga = gru_actor.c if gru_actor is not None else None
    ca = actor.c if actor is not None else None
    return lib.rslx_act_recurrent_workspace_bytes(_ref(ga), _ref(ca), _ref(gru_critic.c), _ref(critic.c), N)


def rslx_act_recurrent(gru_actor, actor, gru_critic, critic, obs_actor, obs_critic, N, h_actor, h_critic, reset, h0_actor_out,
                       h0_critic_out, seed, step, eps, actions, logp, values, mu, sigma, flags, ws):
    ga = gru_actor.c if gru_actor is not None else None
    ca = actor.c if actor is not None else None
    _check(lib.rslx_act_recurrent(_ref(ga), _ref(ca), _ref(gru_critic.c), _ref(critic.c), _ptr(obs_actor), _ptr(obs_critic), N,
                                  _ptr(h_actor), _ptr(h_critic), _ptr(reset), _ptr(h0_actor_out), _ptr(h0_critic_out), seed,
                                  step, _ptr(eps), _ptr(actions), _ptr(logp), _ptr(values), _ptr(mu), _ptr(sigma), flags,
                                  _ptr(ws), ws.numel() if ws is not None else 0, _stream()), "rslx_act_recurrent")


def rslx_act_recurrent_dc(gru_actor, actor, gru_critic, critic, obs_actor, obs_critic, N, h_actor, h_critic, reset, h0_actor_out,
                          h0_critic_out, seed, counters, eps, actions, logp, values, mu, sigma, flags, ws):
    ga = gru_actor.c if gru_actor is not None else None
    ca = actor.c if actor is not None else None
    _check(lib.rslx_act_recurrent_dc(_ref(ga), _ref(ca), _ref(gru_critic.c), _ref(critic.c), _ptr(obs_actor), _ptr(obs_critic), N,
                                     _ptr(h_actor), _ptr(h_critic), _ptr(reset), _ptr(h0_actor_out), _ptr(h0_critic_out), seed,
                                     _ptr(counters), _ptr(eps), _ptr(actions), _ptr(logp), _ptr(values), _ptr(mu), _ptr(sigma),
                                     flags, _ptr(ws), ws.numel() if ws is not None else 0, _stream()), "rslx_act_recurrent_dc")


def rslx_ppo_update_recurrent_dc(gru_actor, actor, gru_critic, critic, rollout, dones, h0_actor, h0_critic, cfg, counters, stats, ws):
    _check(lib.rslx_ppo_update_recurrent_dc(_ref(gru_actor.c), _ref(actor.c), _ref(gru_critic.c), _ref(critic.c), _ref(rollout.c),
                                            _ptr(dones), _ptr(h0_actor), _ptr(h0_critic), _ref(cfg.c), _ptr(counters),
                                            _ptr(stats), _ptr(ws), ws.numel() if ws is not None else 0, _stream()),
           "rslx_ppo_update_recurrent_dc")


def rslx_ppo_update_recurrent_workspace_bytes(gru_actor, actor, gru_critic, critic, rollout, cfg):
    n = lib.rslx_ppo_update_recurrent_workspace_bytes(_ref(gru_actor.c), _ref(actor.c), _ref(gru_critic.c), _ref(critic.c),
                                                      _ref(rollout.c), _ref(cfg.c))
    if n == 0:
        raise RslxError("rslx_ppo_update_recurrent_workspace_bytes: %s" % lib.rslx_last_error().decode())
    return n


def rslx_ppo_update_recurrent(gru_actor, actor, gru_critic, critic, rollout, dones, h0_actor, h0_critic, cfg, adam_step, stats, ws):
    """adam_step: ctypes.c_int64, updated in place."""
    _check(lib.rslx_ppo_update_recurrent(_ref(gru_actor.c), _ref(actor.c), _ref(gru_critic.c), _ref(critic.c), _ref(rollout.c),
                                         _ptr(dones), _ptr(h0_actor), _ptr(h0_critic), _ref(cfg.c), C.byref(adam_step),
                                         _ptr(stats), _ptr(ws), ws.numel() if ws is not None else 0, _stream()),
           "rslx_ppo_update_recurrent")


def rslx_memory_step_workspace_bytes(mem, N):
    return lib.rslx_memory_step_workspace_bytes(_ref(mem.c), N)


def rslx_memory_step(mem, obs, N, state, reset, s0_out, h_dense_out, ws):
    _check(lib.rslx_memory_step(_ref(mem.c), _ptr(obs), N, _ptr(state), _ptr(reset), _ptr(s0_out), _ptr(h_dense_out), _ptr(ws),
                                ws.numel() if ws is not None else 0, _stream()), "rslx_memory_step")


def rslx_bc_update_recurrent_workspace_bytes(gru, student, T, N, cfg):
    n = lib.rslx_bc_update_recurrent_workspace_bytes(_ref(gru.c), _ref(student.c), T, N, _ref(cfg.c))
    if n == 0:
        raise RslxError("rslx_bc_update_recurrent_workspace_bytes: %s" % lib.rslx_last_error().decode())
    return n


def rslx_bc_update_recurrent(gru, student, obs_student, targets, dones, h0, T, N, cfg, adam_step, stats, ws):
    """adam_step: ctypes.c_int64, updated in place."""
    _check(lib.rslx_bc_update_recurrent(_ref(gru.c), _ref(student.c), _ptr(obs_student), _ptr(targets), _ptr(dones), _ptr(h0),
                                        T, N, _ref(cfg.c), C.byref(adam_step), _ptr(stats), _ptr(ws),
                                        ws.numel() if ws is not None else 0, _stream()), "rslx_bc_update_recurrent")


def rslx_sym_augment(sym, obs_in, act_in, B, D, A, obs_out, act_out):
    cs = sym.c
    _check(lib.rslx_sym_augment(_ref(cs), _ptr(obs_in), _ptr(act_in), B, D, A, _ptr(obs_out), _ptr(act_out), _stream()),
           "rslx_sym_augment")


def rslx_rnd_workspace_bytes(target, N):
    return lib.rslx_rnd_workspace_bytes(_ref(target.c), N)


def rslx_rnd(target, predictor, obs, N, D, subset_idx, n_subset, running, weight, update_stats, r_int_out, rewards_inout, ws):
    ct, cp = target.c, predictor.c
    _check(lib.rslx_rnd(_ref(ct), _ref(cp), _ptr(obs), N, D, _ptr(subset_idx), n_subset, _ptr(running), weight,
                        int(update_stats), _ptr(r_int_out), _ptr(rewards_inout), _ptr(ws), ws.numel(), _stream()), "rslx_rnd")


def rslx_trace_begin(max_records):
    _check(lib.rslx_trace_begin(max_records), "rslx_trace_begin")


def rslx_trace_end():
    """Returns [(kernel, flops, bytes, ms)] in launch order."""
    n = C.c_int32(0)
    _check(lib.rslx_trace_end(None, 0, C.byref(n)), "rslx_trace_end")
    buf = (_CTraceRecord * max(n.value, 1))()
    _check(lib.rslx_trace_end(buf, n.value, C.byref(n)), "rslx_trace_end")
    return [(buf[i].kernel.decode(), buf[i].flops, buf[i].bytes, buf[i].ms) for i in range(n.value)]
