"""Pins for oracle.rng: published SplitMix64 vectors, a big-int reimplementation, bijection, moments."""
import os
import numpy as np
from oracle import rng

MASK = (1 << 64) - 1


def mix64_bigint(x):
    x = (x + 0x9E3779B97F4A7C15) & MASK
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & MASK
    return x ^ (x >> 31)


def test_published_splitmix64_vectors(golden_dir):
    want = [int(l, 16) for l in open(os.path.join(golden_dir, "splitmix64_seed0.txt")) if l.startswith("0x")]
    got = [int(rng.mix64(np.uint64((k * 0x9E3779B97F4A7C15) & MASK))) for k in range(3)]
    assert got == want


def test_mix64_matches_bigint():
    xs = [0, 1, 2, 0xFFFFFFFFFFFFFFFF, 0x8000000000000000, 123456789123456789, 20250910]
    got = rng.mix64(np.array(xs, dtype=np.uint64))
    assert [int(g) for g in got] == [mix64_bigint(x) for x in xs]


def perm_bigint(seed, call, epoch, B):
    base = mix64_bigint(mix64_bigint(mix64_bigint(seed) ^ call) ^ epoch)
    keys = [mix64_bigint(base ^ i) for i in range(B)]
    return [i for _, i in sorted(zip(keys, range(B)))]


def test_permutation_matches_bigint_argsort():
    for (seed, call, epoch, B) in [(0, 0, 0, 1), (7, 3, 2, 257), (20250910, 1, 4, 4096)]:
        assert rng.permutation(seed, call, epoch, B).tolist() == perm_bigint(seed, call, epoch, B)


def test_permutation_is_bijection_and_varies():
    B = 1536
    p = rng.permutation(5, 0, 0, B)
    assert p.dtype == np.int32 and sorted(p.tolist()) == list(range(B))
    assert np.array_equal(p, rng.permutation(5, 0, 0, B))
    for other in [(6, 0, 0), (5, 1, 0), (5, 0, 1)]:
        assert not np.array_equal(p, rng.permutation(*other, B))
    # minibatches partition the index set
    mb = B // 4
    assert sorted(np.concatenate([p[m * mb:(m + 1) * mb] for m in range(4)]).tolist()) == list(range(B))


def test_act_noise_bits_and_moments():
    N, A = 100000, 10
    eps = rng.act_noise(11, 3, N, A)
    assert eps.shape == (N, A) and np.all(np.isfinite(eps))
    assert abs(eps.mean()) < 5e-3 and abs(eps.var() - 1.0) < 1e-2
    assert abs(np.mean(eps ** 3)) < 2e-2 and abs(np.mean(eps ** 4) - 3.0) < 6e-2
    # one element recomputed with python integers / math
    import math
    n, j = 1234, 7
    base = mix64_bigint(mix64_bigint(11 ^ 0xAC7) ^ 3)
    h = mix64_bigint(base ^ (n * A + j))
    u1 = ((h >> 40) + 1) / 2 ** 24
    u2 = ((h >> 8) & 0xFFFFFF) / 2 ** 24
    assert 0 < u1 <= 1 and 0 <= u2 < 1
    assert abs(eps[n, j] - math.sqrt(-2 * math.log(u1)) * math.cos(2 * math.pi * u2)) < 1e-14
    assert not np.array_equal(eps, rng.act_noise(11, 4, N, A))
