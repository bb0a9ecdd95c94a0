"""Counter-based random numbers of the method: minibatch permutations and action noise.

The paper states PPO with "multi-epoch minibatch" updates (Sec. 2.1) and gives no
generator, so the generator is this repository's own definition, built on the
published SplitMix64 finaliser (Steele, Lea, Flood 2014):

    mix64(x):  x += 0x9E3779B97F4A7C15
               x  = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9
               x  = (x ^ (x >> 27)) * 0x94D049BB133111EB
               return x ^ (x >> 31)                    (all mod 2^64)

Oracle code: test infrastructure only.
"""
import numpy as np

_U = np.uint64
_GOLD = _U(0x9E3779B97F4A7C15)
_M1 = _U(0xBF58476D1CE4E5B9)
_M2 = _U(0x94D049BB133111EB)
ACT_SALT = 0xAC7


def mix64(x):
    """SplitMix64 output function applied to x (scalar or array), mod 2^64."""
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        x = x + _GOLD
        x = (x ^ (x >> _U(30))) * _M1
        x = (x ^ (x >> _U(27))) * _M2
        return x ^ (x >> _U(31))


def permutation_keys(seed, call_index, epoch, B):
    """key_i = mix64(mix64(mix64(mix64(seed) ^ call) ^ epoch) ^ i), i in [0, B)."""
    base = mix64(mix64(mix64(_U(seed)) ^ _U(call_index)) ^ _U(epoch))
    return mix64(base ^ np.arange(B, dtype=np.uint64))


def permutation(seed, call_index, epoch, B):
    """Indices [0, B) sorted ascending by (key_i, i): the shuffled order of one epoch.

    A stable sort on key alone gives exactly the (key, i) lexicographic order.
    """
    keys = permutation_keys(seed, call_index, epoch, B)
    return np.argsort(keys, kind="stable").astype(np.int32)


def act_noise(seed, step, N, A):
    """Standard-normal noise eps[n, j] for act() at rollout step `step`.

    h  = mix64(mix64(mix64(seed ^ 0xAC7) ^ step) ^ (n*A + j))
    u1 = ((h >> 40) + 1) * 2^-24   in (0, 1]
    u2 = ((h >> 8) & 0xFFFFFF) * 2^-24   in [0, 1)
    eps = sqrt(-2 ln u1) * cos(2 pi u2)          (Box-Muller, cosine branch)
    """
    base = mix64(mix64(_U(seed) ^ _U(ACT_SALT)) ^ _U(step))
    h = mix64(base ^ np.arange(N * A, dtype=np.uint64))
    u1 = ((h >> _U(40)).astype(np.float64) + 1.0) * 2.0 ** -24
    u2 = ((h >> _U(8)) & _U(0xFFFFFF)).astype(np.float64) * 2.0 ** -24
    eps = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return eps.reshape(N, A)
