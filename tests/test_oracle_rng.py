"""Pins for the oracle's branch draw b_k^(t) (Alg. 1: b ~ U[0,1], mix iff b <= p; App. A.2:
independent Bernoulli(p) per worker and step).  The generator is the SplitMix64 output
function used as a counter hash; its published reference outputs are the fixture."""
import math
import os

import numpy as np

M64 = 2 ** 64
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_seed0.txt")


def _bigint_hash(seed, idx):
    z = (seed + (idx + 1) * 0x9E3779B97F4A7C15) % M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) % M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) % M64
    return z ^ (z >> 31)


def test_published_vectors(oracle_mod):
    vals = [int(l, 16) for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(vals) >= 4
    for n, v in enumerate(vals):
        # idx = t*K + k = n with K = 1, and with K = 4 (t = n // 4, k = n % 4)
        assert oracle_mod.u24(0, n, 0, 1) == v >> 40
        assert oracle_mod.u24(0, n // 4, n % 4, 4) == v >> 40


def test_against_bigint_formula(oracle_mod):
    rng = np.random.default_rng(7)
    for _ in range(1000):
        seed = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
        K = int(rng.integers(1, 65))
        k = int(rng.integers(0, K))
        t = int(rng.integers(0, 2 ** 40))
        assert oracle_mod.u24(seed, t, k, K) == _bigint_hash(seed, t * K + k) >> 40


def test_threshold_rule(oracle_mod):
    # mix iff u24 < floor(p * 2^24): p = 0 never mixes, p -> 1 almost always
    for t in range(200):
        assert oracle_mod.draw(3, t, 1, 4, 0.0) == 0
        u = oracle_mod.u24(3, t, 1, 4)
        for p in (0.02, 0.05, 0.1, 0.25, 0.5, 0.999):
            assert oracle_mod.draw(3, t, 1, 4, p) == int(u < math.floor(p * 2 ** 24))
    # exact grid point: p = j / 2^24 mixes exactly the u24 values below j
    j = oracle_mod.u24(11, 5, 2, 8)
    assert oracle_mod.draw(11, 5, 2, 8, j / 2 ** 24) == 0
    assert oracle_mod.draw(11, 5, 2, 8, (j + 1) / 2 ** 24) == 1


def test_frequency_and_independence(oracle_mod):
    K, T = 8, 20000
    for p in (0.02, 0.05, 0.1, 0.25):
        b = np.array([[oracle_mod.draw(2024, t, k, K, p) for k in range(K)] for t in range(T)], float)
        n = b.size
        assert abs(b.mean() - p) < 4 * math.sqrt(p * (1 - p) / n)
        # per-worker frequencies and lag-1 / cross-worker correlations are those of independent draws
        for k in range(K):
            assert abs(b[:, k].mean() - p) < 4.5 * math.sqrt(p * (1 - p) / T)
        c = b - p
        lag = (c[1:] * c[:-1]).mean() / (p * (1 - p))
        cross = (c[:, 0] * c[:, 1]).mean() / (p * (1 - p))
        assert abs(lag) < 5 / math.sqrt(n) and abs(cross) < 5 / math.sqrt(T)
