"""Pins for the oracle's synthetic-gradient generator (CPU only).

The generator stands in for the gradient computation step of Alg. B
with a counter-based stream, so it is pinned against things other than itself:
published known-answer vectors, an independent big-integer transcription of the
published round function, libm, and distribution tests against scipy.
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

from paper_2103_07454_amd import inputs

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def philox_bigint(ctr, key):
    """Philox4x32-10 with Python integers, written from the SC'11 description."""
    M0, M1, W0, W1, MASK = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85, 0xFFFFFFFF
    c = [int(v) for v in ctr]
    k = [int(v) for v in key]
    for rnd in range(10):
        if rnd:
            k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
        p0, p1 = M0 * c[0], M1 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & MASK, (p0 >> 32) ^ c[3] ^ k[1], p0 & MASK]
    return c


def test_philox_known_answers(oracle_mod):
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        v = [int(t, 16) for t in row]
        got = oracle_mod.philox4x32_10(v[0:4], v[4:6])
        assert [int(g) for g in got] == v[6:10]
        assert philox_bigint(v[0:4], v[4:6]) == v[6:10]


def test_philox_matches_bigint_on_random_counters(oracle_mod):
    rng = np.random.default_rng(7)
    for _ in range(2000):
        ctr = rng.integers(0, 2**32, 4, dtype=np.uint64)
        key = rng.integers(0, 2**32, 2, dtype=np.uint64)
        assert [int(g) for g in oracle_mod.philox4x32_10(ctr, key)] == philox_bigint(ctr, key)


def test_uniform_is_exact_and_open(oracle_mod):
    from fractions import Fraction
    for w in [0, 1, 511, 512, 2**31, 2**32 - 1, 0x12345678]:
        u = oracle_mod.uniform01(w)
        assert Fraction(u) == (Fraction(w >> 9) + Fraction(1, 2)) / 2**23
        assert 0.0 < u < 1.0


def test_log_polynomial_against_libm(oracle_mod):
    rng = np.random.default_rng(3)
    us = np.concatenate([rng.random(20000).astype(np.float32),
                         np.float32(2.0) ** -rng.integers(1, 24, 2000).astype(np.float32)
                         * (1 + rng.random(2000).astype(np.float32)) / 2,
                         np.array([2.0**-24, 1 - 2.0**-24, 0.5, 0.70710677, 0.7071068], np.float32)])
    us = us[(us > 0) & (us < 1)]
    for u in us:
        ref = math.log(float(u))
        assert abs(oracle_mod.log_poly(u) - ref) <= 3e-7 * abs(ref) + 2e-8


def test_exp_polynomial_against_libm(oracle_mod):
    rng = np.random.default_rng(6)
    ys = np.concatenate([rng.random(20000).astype(np.float32) * np.float32(11.2),
                         np.float32(2.0) ** -rng.integers(1, 30, 2000).astype(np.float32),
                         np.array([0.0, 0.34657359, 0.346574, 0.6931472, 11.09, 1e-8], np.float32)])
    for y in ys:
        ref = math.exp(float(y))
        assert abs(oracle_mod.exp_poly(y) - ref) <= 4e-7 * ref
    assert oracle_mod.exp_poly(0.0) == 1.0


def test_sincos_polynomial_against_libm(oracle_mod):
    us = np.concatenate([np.random.default_rng(4).random(20000).astype(np.float32),
                         np.arange(0, 1, 1 / 64, dtype=np.float32),
                         np.array([1 - 2.0**-24], np.float32)])
    for u in us:
        c, s = oracle_mod.sincos2pi(u)
        assert abs(c - math.cos(2 * math.pi * float(u))) < 3e-7
        assert abs(s - math.sin(2 * math.pi * float(u))) < 3e-7
        assert abs(c * c + s * s - 1) < 5e-7


def test_box_muller_pairs(oracle_mod):
    """z0,z1 come from words 0,1 and z2,z3 from words 2,3: radius from the first
    word of each pair, angle from the second."""
    rng = np.random.default_rng(5)
    for _ in range(500):
        w = rng.integers(0, 2**32, 4, dtype=np.uint64)
        z = oracle_mod.normal4(w)
        for h in range(2):
            ua = (int(w[2 * h]) >> 9) + 0.5
            ub = (int(w[2 * h + 1]) >> 9) + 0.5
            rad = math.sqrt(-2 * math.log(ua / 2**23))
            ang = 2 * math.pi * ub / 2**23
            assert abs(z[2 * h] - rad * math.cos(ang)) < 2e-6
            assert abs(z[2 * h + 1] - rad * math.sin(ang)) < 2e-6


def _orc(oracle_mod, tensors, P=3, **kw):
    numel = np.array([t.numel for t in tensors], np.uint64)
    fan = np.array([t.fan_in for t in tensors], np.uint32)
    x0 = np.zeros((P, int(numel.sum())), np.float32)
    return oracle_mod.Oracle(x0, numel, fan, **kw)


def test_counter_layout(oracle_mod):
    """counter = (index/4, tensor, iteration, worker), key = seed halves; element j
    takes output j%4 of its block (normal case); one block per element for
    Student-t."""
    tensors = inputs.mlp((6, 5, 3))
    seed = 0x0123456789ABCDEF
    key = [seed & 0xFFFFFFFF, seed >> 32]
    o = _orc(oracle_mod, tensors, P=4, seed=seed, sigma0=1.0)
    for (r, k, l) in [(0, 0, 0), (3, 17, 2), (1, 5, 1)]:
        g = o.grad_tensor(r, k, l)
        for j in range(g.size):
            z = oracle_mod.normal4(philox_bigint([j // 4, l, k, r], key))
            assert g[j] == z[j % 4]
    # Student-t(3), polar method: elements 4g .. 4g+3 share Philox blocks 2g, 2g+1; element 4g+i takes
    # word 2i for the radius, R^2 = 3 (u^(-2/3) - 1), and word 2i+1 for the angle
    ot = _orc(oracle_mod, tensors, P=4, seed=seed, sigma0=1.0, dist=1)
    for (r, k, l) in [(2, 9, 0), (0, 0, 1), (3, 4, 2)]:
        g = ot.grad_tensor(r, k, l)
        for j in range(g.size):
            words = philox_bigint([2 * (j // 4), l, k, r], key) + philox_bigint([2 * (j // 4) + 1, l, k, r], key)
            i = j % 4
            u, v = (((w >> 9) + 0.5) / 2**23 for w in words[2 * i:2 * i + 2])
            want = math.sqrt(3 * (u ** (-2 / 3) - 1)) * math.cos(2 * math.pi * v)
            assert abs(g[j] - want) < 2e-5 * max(1, abs(want)) + 2e-4, (r, k, l, j)


def test_normal_distribution(oracle_mod):
    tensors = [inputs.TensorSpec("w", (1 << 20,), 64, "weight")]
    o = _orc(oracle_mod, tensors, seed=11, sigma0=1.0)
    g = o.grad_tensor(1, 3, 0).astype(np.float64)
    n = g.size
    assert abs(g.mean()) < 4 / math.sqrt(n)
    assert abs(g.std() - 1) < 4 / math.sqrt(2 * n)
    assert stats.kstest(g, "norm").pvalue > 1e-3
    assert abs(stats.kurtosis(g)) < 0.03
    # neighbours in a block and across blocks are uncorrelated
    assert abs(np.corrcoef(g[0::4], g[1::4])[0, 1]) < 0.01
    assert abs(np.corrcoef(g[:-4], g[4:])[0, 1]) < 0.01


def test_student_t_distribution(oracle_mod):
    tensors = [inputs.TensorSpec("w", (1 << 18,), 64, "weight")]
    o = _orc(oracle_mod, tensors, seed=12, sigma0=1.0, dist=1)
    g = o.grad_tensor(0, 0, 0).astype(np.float64)
    assert stats.kstest(g, "t", args=(3,)).pvalue > 1e-3
    assert abs(np.quantile(g, 0.75) - stats.t.ppf(0.75, 3)) < 0.01   # ~0.765
    assert abs(np.quantile(g, 0.99) - stats.t.ppf(0.99, 3)) < 0.15   # ~4.54: the heavy tail is there
    assert abs(np.median(g)) < 0.01
    # variates that share Philox blocks are uncorrelated (signs and magnitudes)
    for a, b in ((g[0::4], g[1::4]), (g[1::4], g[2::4]), (g[:-4:4], g[4::4])):
        assert abs(np.corrcoef(np.sign(a), np.sign(b))[0, 1]) < 0.02
        assert abs(stats.spearmanr(np.abs(a), np.abs(b)).statistic) < 0.02


def test_sigma_fan_in_decay_and_spike(oracle_mod):
    tensors = [inputs.TensorSpec("a", (40000,), 16, "weight"),
               inputs.TensorSpec("b", (40000,), 400, "weight")]
    o = _orc(oracle_mod, tensors, P=8, seed=13, sigma0=0.02, fan_in_scaling=1, decay=0.9)
    for l, fan in ((0, 16), (1, 400)):
        for k in (0, 10):
            g = o.grad_tensor(0, k, l).astype(np.float64)
            want = 0.02 / math.sqrt(fan) * 0.9**k
            assert abs(g.std() / want - 1) < 0.02
    flat = _orc(oracle_mod, tensors, P=8, seed=13, sigma0=0.02, fan_in_scaling=0, decay=1.0)
    assert abs(flat.grad_tensor(0, 5, 1).astype(np.float64).std() / 0.02 - 1) < 0.02
    # spikes multiply a whole (worker, iteration) gradient by the gain, with the given probability
    sp = _orc(oracle_mod, tensors, P=8, seed=13, sigma0=0.02, fan_in_scaling=1, decay=0.9,
              spike_prob=0.1, spike_gain=5.0)
    hits = 0
    total = 0
    for r in range(8):
        for k in range(60):
            a = o.grad_tensor(r, k, 0)[:64]
            b = sp.grad_tensor(r, k, 0)[:64]
            b1 = sp.grad_tensor(r, k, 1)[:64]
            a1 = o.grad_tensor(r, k, 1)[:64]
            if np.array_equal(a, b):
                assert np.array_equal(a1, b1)
            else:
                assert np.array_equal(a * np.float32(5), b) and np.array_equal(a1 * np.float32(5), b1)
                hits += 1
            total += 1
    assert 0.05 < hits / total < 0.16


def test_streams_differ_by_worker_iteration_tensor_seed(oracle_mod):
    tensors = [inputs.TensorSpec("a", (64,), 1, "weight"), inputs.TensorSpec("b", (64,), 1, "weight")]
    o = _orc(oracle_mod, tensors, P=3, seed=1, sigma0=1.0)
    o2 = _orc(oracle_mod, tensors, P=3, seed=2, sigma0=1.0)
    base = o.grad_tensor(0, 0, 0)
    for other in (o.grad_tensor(1, 0, 0), o.grad_tensor(0, 1, 0), o.grad_tensor(0, 0, 1),
                  o2.grad_tensor(0, 0, 0)):
        assert not np.any(base == other)
    assert np.array_equal(base, o.grad_tensor(0, 0, 0))
