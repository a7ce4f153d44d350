"""Pins for the parts of the oracle that concern precision and bookkeeping (CPU only):
double-precision norm accumulation, the width and strictness of the near-tie band, where
spikes fall, and the message fingerprints.  Each expected value is computed here from first
principles (exact rational / big-integer / math.fsum arithmetic), never by the oracle."""
import math
from fractions import Fraction

import numpy as np
import pytest

from paper_2103_07454_amd import inputs

from test_oracle_generator import philox_bigint

INF = float("inf")


def one_tensor_ring(oracle_mod, drift, P=3, **kw):
    """P workers, one tensor, x0 = 0 (so xhat = 0) and x := drift for every worker: the drift
    x - xhat is then exactly `drift`.  Nothing ever fires unless kw says so."""
    drift = np.asarray(drift, np.float32)
    n = drift.size
    base = dict(thr_mode=0, thr_fixed=INF, force_first=0, lr=0.0, momentum=0.0, sigma0=0.0)
    base.update(kw)
    o = oracle_mod.Oracle(np.zeros((P, n), np.float32), [n], None, **base)
    o.set_state("x", np.broadcast_to(drift, (P, n)))
    return o


# ---------------------------------------------------------------------------------------
# the drift norm is accumulated in double precision and rounded to float once
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("trigger_kind", [0, 1])
def test_norm_is_accumulated_in_double(oracle_mod, trigger_kind):
    # one drift of 1 followed by 2^22 drifts of 2^-13: every later square (2^-26) is below half
    # an ulp of the running float sum, so float accumulation in index order stays at 1.0 and
    # misses the true 1 + 2^-4 by 3 %.  Pairwise or blocked float sums get closer but not exact;
    # the double sum is exact here, so the norm must be sqrt(1.0625) rounded once.
    n = (1 << 22) + 1
    drift = np.full(n, 2.0 ** -13, np.float32)
    drift[0] = 1.0
    o = one_tensor_ring(oracle_mod, drift, trigger_kind=trigger_kind)
    o.step(0)
    exact = Fraction(1) + (n - 1) * Fraction(1, 2 ** 26)      # sum of the squared drifts
    assert exact == Fraction(17, 16)
    want = np.float32(math.sqrt(float(exact)))
    d = o.decisions()
    assert (d["norm"] == want).all(), (d["norm"], want)
    assert abs(float(want) - 1.0) > 1e-2      # float accumulation would have returned exactly 1.0


def test_norm_against_exact_rational_sum_on_random_drift(oracle_mod):
    # values spanning 12 binades: the exact sum of squares as a rational, its square root
    # rounded once to float (double sqrt of the correctly rounded double sum differs from that
    # by far less than the 2e-7 the GPU comparison allows; here the two agree exactly)
    rng = np.random.default_rng(21)
    drift = (rng.standard_normal(5000) * 2.0 ** rng.integers(-6, 6, 5000)).astype(np.float32)
    o = one_tensor_ring(oracle_mod, drift)
    o.step(0)
    exact = sum(Fraction(float(v)) ** 2 for v in drift)
    want = np.float32(math.sqrt(float(exact)))
    got = o.decisions()["norm"][0, 0]
    assert got == want or abs(float(got) - math.sqrt(float(exact))) <= 0.5000001 * float(np.spacing(want))


# ---------------------------------------------------------------------------------------
# the near-tie band: |norm - delta| < 1e-6 * delta, strictly, in float arithmetic
# ---------------------------------------------------------------------------------------
def band_case(oracle_mod, delta, norms):
    """One single-element tensor per norm value, all tested against the fixed threshold delta."""
    norms = np.asarray(norms, np.float32)
    L = norms.size
    o = oracle_mod.Oracle(np.zeros((3, L), np.float32), [1] * L, None, thr_mode=0, thr_fixed=float(delta),
                          force_first=0, lr=0.0, momentum=0.0, sigma0=0.0)
    o.set_state("x", np.broadcast_to(norms, (3, L)))
    o.step(0)
    d = o.decisions()
    assert np.array_equal(d["norm"][0], norms)          # a one-element drift is its own norm
    return d["near_tie"][0].astype(bool), d["fired"][0] > 0, o.totals()["near_tie_flags"]


def test_near_tie_band_width_and_strictness(oracle_mod):
    u = 2.0 ** -23                                     # spacing of floats in [1, 2); half of it below 1
    norms = [1 + 8 * u,       # +9.54e-7: inside
             1 + 9 * u,       # +1.073e-6: outside
             1 - 16 * u / 2,  # -9.54e-7: inside
             1 - 18 * u / 2,  # -1.073e-6: outside
             1.0,             # the tie itself: inside (and it fires: >=)
             1 + u, 1 - u / 2, 0.5, 2.0, 0.0]
    near, fired, count = band_case(oracle_mod, 1.0, norms)
    assert near.tolist() == [True, False, True, False, True, True, True, False, False, False]
    assert fired.tolist() == [True, True, False, False, True, True, False, False, True, False]
    assert count == 3 * 5                              # counted once per flagged test, three workers


def test_near_tie_band_boundary_is_excluded(oracle_mod):
    # delta = 2^-126 (smallest normal float): 1e-6f * delta = 8.39 units of 2^-149 rounds to 8
    # units, and |norm - delta| is a whole number of units, so equality with the band's edge
    # can be met exactly: 7 units inside, 8 units ON the edge = outside (strict <), 9 outside
    unit = 2.0 ** -149
    delta = 2.0 ** -126
    assert np.float32(1e-6) * np.float32(delta) == np.float32(8 * unit)
    near, fired, count = band_case(oracle_mod, delta, [delta + 7 * unit, delta + 8 * unit, delta + 9 * unit,
                                                       delta - 7 * unit, delta - 8 * unit, delta])
    assert near.tolist() == [True, False, False, True, False, True]
    assert fired.tolist() == [True, True, True, False, False, True]
    assert count == 3 * 3


def test_near_tie_band_is_empty_for_zero_and_infinite_thresholds(oracle_mod):
    near, fired, count = band_case(oracle_mod, 0.0, [0.0, 2.0 ** -149, 1.0])
    assert not near.any() and fired.all() and count == 0           # 0 >= 0 fires, never a "near" tie
    near, fired, count = band_case(oracle_mod, INF, [0.0, 1.0, 3.0e38])
    assert not near.any() and not fired.any() and count == 0


def test_adaptive_near_tie_uses_the_threshold_before_the_event(oracle_mod):
    # adaptive threshold, one element: the band is judged against the delta the norm was
    # compared with, not the one recomputed at the event
    o = oracle_mod.Oracle(np.zeros((3, 1), np.float32), [1], None, thr_mode=1, delta_init=1.0, horizon=1.0,
                          force_first=0, lr=0.0, momentum=0.0, sigma0=0.0)
    o.set_state("x", np.full((3, 1), 1 + 4 * 2.0 ** -23, np.float32))
    o.step(0)
    d = o.decisions()
    assert d["near_tie"].all() and (d["fired"] == 1).all() and (d["delta_before"] == 1.0).all()
    assert o.totals()["near_tie_flags"] == 3


# ---------------------------------------------------------------------------------------
# spikes: the draw of (worker, iteration) uses counter (0, 0xFFFFFFFF, k, r), word 0
# ---------------------------------------------------------------------------------------
def test_spikes_fall_where_the_reserved_counter_says(oracle_mod):
    seed = 0x00C0FFEE12345678
    key = [seed & 0xFFFFFFFF, seed >> 32]
    P, prob, gain = 5, 0.25, 3.0
    numel = np.array([8, 5], np.uint64)
    x0 = np.zeros((P, 13), np.float32)
    plain = oracle_mod.Oracle(x0, numel, None, seed=seed, sigma0=1.0)
    spiky = oracle_mod.Oracle(x0, numel, None, seed=seed, sigma0=1.0, spike_prob=prob, spike_gain=gain)
    hits = 0
    for r in range(P):
        for k in range(40):
            w0 = philox_bigint([0, 0xFFFFFFFF, k, r], key)[0]
            u = Fraction((w0 >> 9) * 2 + 1, 2 ** 24)            # ((w >> 9) + 1/2) / 2^23, exactly
            want_spike = u < Fraction(float(np.float32(prob)))
            hits += want_spike
            for l in range(2):
                a, b = plain.grad_tensor(r, k, l), spiky.grad_tensor(r, k, l)
                if want_spike:
                    assert np.array_equal(b, a * np.float32(gain)) and not np.array_equal(a, b), (r, k, l)
                else:
                    assert np.array_equal(a, b), (r, k, l)
    assert 30 <= hits <= 70                                     # 200 draws at probability 1/4


# ---------------------------------------------------------------------------------------
# message fingerprints
# ---------------------------------------------------------------------------------------
def splitmix64_bigint(z):
    M = (1 << 64) - 1
    z = (z + 0x9E3779B97F4A7C15) & M
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
    return z ^ (z >> 31)


def test_splitmix64_known_answer_and_bigint(oracle_mod):
    # first output of the SplitMix64 generator seeded with 0, as published with the generator
    assert oracle_mod.splitmix64(0) == 0xE220A8397B1DCDAF
    rng = np.random.default_rng(8)
    for z in [1, 2 ** 32, 2 ** 64 - 1] + [int(v) for v in rng.integers(0, 2 ** 63, 200)]:
        assert oracle_mod.splitmix64(z) == splitmix64_bigint(z)


def test_message_fingerprints_are_sums_over_the_message(oracle_mod):
    tensors = [inputs.TensorSpec("a", (700,), 4, "weight"), inputs.TensorSpec("b", (3,), 4, "bias"),
               inputs.TensorSpec("c", (90,), 4, "weight")]
    w = inputs.Workload("fp", 4, tensors, 8, sigma0=0.05, decay=0.97, topk_ppm=100_000, seed=5)
    o = oracle_mod.Oracle.from_workload(w)
    M = (1 << 64) - 1
    seen = 0
    for k in range(8):
        o.step(k)
        fired = o.decisions()["fired"]
        ih, mh = o.message_hashes()
        for r in range(w.P):
            for l in range(w.L):
                idx, val = o.message(r, l)
                if fired[r, l] != 2:
                    assert idx.size == 0 and ih[r, l] == 0 and mh[r, l] == 0
                    continue
                seen += 1
                bits = val.view(np.uint32)
                assert int(ih[r, l]) == sum(splitmix64_bigint(int(j)) for j in idx) & M
                assert int(mh[r, l]) == sum(splitmix64_bigint((int(b) << 32) | int(j)) for j, b in zip(idx, bits)) & M
    assert seen > 20
