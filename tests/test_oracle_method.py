"""Pins for the oracle's trigger / send / averaging / update steps (CPU only).

Every test checks the oracle against something the paper or the mathematics
fixes independently of the oracle's own code: a dense mixing-matrix form of
Eq. 2, closed forms of a scalar toy problem, brute-force selection, invariants
of Sections 3-5, or limits in which the scheme degenerates to plain SGD.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from paper_2103_07454_amd import inputs

INF = float("inf")


def ring_matrix(P):
    """Symmetric doubly-stochastic ring matrix with weights 1/3 (Section 3)."""
    W = np.zeros((P, P))
    for i in range(P):
        for j in (i - 1, i, i + 1):
            W[i, j % P] += 1.0 / 3.0
    return W


def make(oracle_mod, numel, P, x0=None, seed=1, **kw):
    numel = np.asarray(numel, np.uint64)
    n = int(numel.sum())
    if x0 is None:
        x0 = inputs.distinct_params(n, P, seed)
    return oracle_mod.Oracle(x0, numel, np.ones(len(numel), np.uint32), **kw), x0


# --------------------------------------------------------------------------
# threshold 0 is the regular algorithm (Section 5, remark after Corollary 1)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("P", [3, 4, 7])
def test_threshold_zero_is_dense_dpsgd(oracle_mod, P):
    numel = [5, 12, 1, 33]
    n = sum(numel)
    lr, mu = 0.05, 0.9
    o, x0 = make(oracle_mod, numel, P, thr_mode=0, thr_fixed=0.0, lr=lr, momentum=mu, grad_mode=1)
    W = ring_matrix(P)
    X = x0.astype(np.float64).T           # N x n, columns are workers (Section 3)
    V = np.zeros_like(X)
    for k in range(25):
        g = inputs.random_grads(P, n, 100 + k, 0.1)
        o.step(k, grad=g)
        V = mu * V + g.astype(np.float64).T
        X = X @ W - lr * V                # Eq. 2 with the momentum buffer as the gradient term
        assert o.decisions()["fired"].all()
        np.testing.assert_allclose(o.state("x").T, X, rtol=0, atol=2e-6 * np.abs(X).max())
    t = o.totals()
    assert t["events_total"] == P * len(numel) * 25


# --------------------------------------------------------------------------
# infinite threshold, no forced event: P independent momentum-SGD runs, bitwise
# --------------------------------------------------------------------------
def test_threshold_infinite_is_local_sgd_bitwise(oracle_mod):
    numel = [7, 64, 3]
    P, n = 5, sum(numel)
    lr, mu = np.float32(0.05), np.float32(0.9)
    o, x0 = make(oracle_mod, numel, P, thr_mode=0, thr_fixed=INF, force_first=0,
                 lr=float(lr), momentum=float(mu), grad_mode=1)
    x = x0.copy()
    v = np.zeros_like(x)
    for k in range(30):
        g = inputs.random_grads(P, n, 500 + k)
        o.step(k, grad=g)
        # products of two floats are exact in double; one rounding to float32 follows
        v = (mu.astype(np.float64) * v.astype(np.float64) + g.astype(np.float64)).astype(np.float32)
        x = (x.astype(np.float64) - lr.astype(np.float64) * v.astype(np.float64)).astype(np.float32)
        assert not o.decisions()["fired"].any()
    assert np.array_equal(o.state("x"), x)
    assert np.array_equal(o.state("vel"), v)
    assert o.totals()["events_total"] == 0
    tb = o.tables()
    assert not tb["valid_l"].any() and not tb["valid_r"].any()
    assert np.array_equal(o.state("xhat"), x0)


def test_infinite_threshold_with_forced_first_event_anchors_to_x0(oracle_mod):
    """With the paper's forced event at k = 0 the neighbours' copies of x0 keep
    being averaged in, so this is *not* local SGD: documents why the limit above
    needs force_first = 0."""
    numel = [16]
    o, x0 = make(oracle_mod, numel, 4, thr_mode=0, thr_fixed=INF, force_first=1, grad_mode=1,
                 lr=0.1, momentum=0.0)
    g = np.ones((4, 16), np.float32)
    for k in range(3):
        o.step(k, grad=g)
    assert o.totals()["events_total"] == 4          # only the forced ones
    local = x0 - np.float32(0.3)
    assert not np.allclose(o.state("x"), local)


# --------------------------------------------------------------------------
# W 1 = 1: the worker mean is conserved under full communication (Sections 3, 5)
# --------------------------------------------------------------------------
def test_mean_conserved_and_range_contracts_with_zero_gradients(oracle_mod):
    numel = [9, 30]
    P, n = 6, 39
    o, x0 = make(oracle_mod, numel, P, thr_mode=0, thr_fixed=0.0, grad_mode=1, momentum=0.9)
    zero = np.zeros((P, n), np.float32)
    mean0 = x0.astype(np.float64).mean(0)
    spread = np.ptp(x0, axis=0)
    for k in range(40):
        o.step(k, grad=zero)
        x = o.state("x")
        np.testing.assert_allclose(x.astype(np.float64).mean(0), mean0, atol=1e-6)
        new_spread = np.ptp(x, axis=0)
        assert (new_spread <= spread + 1e-6).all()
        spread = new_spread
    assert spread.max() < 0.05 * np.ptp(x0, axis=0).max()   # consensus is reached
    assert not np.any(o.state("vel"))


def test_mean_not_conserved_with_stale_mailboxes(oracle_mod):
    """Property of the method, not a bug: averaging with stale copies does not keep the mean."""
    numel = [8]
    P = 4
    o, x0 = make(oracle_mod, numel, P, thr_mode=0, thr_fixed=0.0, grad_mode=1, momentum=0.0, lr=1.0)
    g = inputs.random_grads(P, 8, 3)
    o.step(0, grad=g)                      # everything is sent once
    o2, _ = make(oracle_mod, numel, P, x0=x0, thr_mode=0, thr_fixed=INF, grad_mode=1, momentum=0.0, lr=1.0)
    o2.step(0, grad=g)                     # forced event at k=0, silence afterwards
    zero = np.zeros_like(g)
    m_after0 = o2.state("x").astype(np.float64).mean(0)
    o2.step(1, grad=zero)
    assert np.abs(o2.state("x").astype(np.float64).mean(0) - m_after0).max() > 1e-3


# --------------------------------------------------------------------------
# scalar toy with closed forms (Eq. 3, trigger with >=, ring averaging)
# --------------------------------------------------------------------------
def scalar_run(oracle_mod, iters, **kw):
    P = 3
    x0 = np.zeros((P, 1), np.float32)
    o = oracle_mod.Oracle(x0, np.array([1], np.uint64), None, lr=0.5, momentum=0.0, grad_mode=1, **kw)
    g = np.ones((P, 1), np.float32)
    rows = []
    for k in range(iters):
        o.step(k, grad=g)
        d = o.decisions()
        rows.append((bool(d["fired"][0, 0]), float(d["norm"][0, 0]), float(o.tables()["delta"][0, 0])))
    return o, rows


def drift_after(m, lr=0.5, c=1.0):
    """|x - xhat| seen by the test m iterations after an event, identical workers,
    constant gradient c: e_{m+1} = e_m/3 - lr c, e_0 = 0  =>  1.5 lr |c| (1 - 3^-m)."""
    return float(Fraction(3, 2) * Fraction(lr) * Fraction(c) * (1 - Fraction(1, 3**m)))


@pytest.mark.parametrize("thr,period", [(0.4, 1), (0.5, 1), (0.6, 2), (0.7, 3), (0.74, 4), (0.8, None)])
def test_fixed_threshold_event_period(oracle_mod, thr, period):
    _, rows = scalar_run(oracle_mod, 40, thr_mode=0, thr_fixed=thr)
    events = [k for k, r in enumerate(rows) if r[0]]
    assert events[0] == 0                               # forced (Section 4)
    if period is None:
        assert events == [0]
        assert abs(rows[-1][1] - 0.75) < 1e-6           # drift saturates at 1.5 lr c
        return
    # closed form: first m with 1.5 lr c (1 - 3^-m) >= thr
    m = next(m for m in range(1, 50) if drift_after(m) >= thr)
    assert m == period
    assert events == list(range(0, 40, period))
    for k in events[1:]:
        assert abs(rows[k][1] - drift_after(period)) < 1e-6


def test_adaptive_threshold_closed_form(oracle_mod):
    # h = 1: an event every iteration, the tie d == delta fires (>=), delta = lr |c|
    _, rows = scalar_run(oracle_mod, 20, thr_mode=1, horizon=1.0)
    assert all(r[0] for r in rows)
    assert rows[0][2] == 0.0 and all(r[2] == 0.5 for r in rows[1:])
    assert all(r[1] == 0.5 for r in rows[1:])
    # h = 2: delta = 2 * 0.5 = 1 after k = 1, never reached again (drift < 0.75)
    _, rows = scalar_run(oracle_mod, 30, thr_mode=1, horizon=2.0)
    assert [k for k, r in enumerate(rows) if r[0]] == [0, 1]
    assert rows[-1][2] == 1.0
    # h = 1.4: delta = 0.7 -> next event 3 iterations later with drift 13/18, then
    # delta = 1.4 * (13/18) / 3 = 0.337 -> next event 1 iteration later, and so on (3,1,3,1,...)
    _, rows = scalar_run(oracle_mod, 30, thr_mode=1, horizon=1.4)
    events = [k for k, r in enumerate(rows) if r[0]]
    assert events[:8] == [0, 1, 4, 5, 8, 9, 12, 13]
    assert abs(rows[1][2] - 0.7) < 1e-6
    assert abs(rows[4][2] - 1.4 * drift_after(3) / 3) < 1e-6
    assert abs(rows[5][2] - 0.7) < 1e-6
    # between events the threshold is held (Section 4, text before Eq. 3)
    assert rows[2][2] == rows[1][2] == rows[3][2]


def test_history_averaged_slope(oracle_mod):
    """Section 7: with a history, the threshold is h times the mean of the slopes
    between consecutive events.  h = 1.4 scalar toy, history of 2."""
    _, rows = scalar_run(oracle_mod, 12, thr_mode=1, horizon=1.4, hist_len=2)
    # event k=0: slope 0 -> delta 0; k=1: slopes (0, .5) -> delta = 1.4*.25 = .35
    assert abs(rows[1][2] - 0.35) < 1e-6
    # k=2 fires (drift .5 >= .35): slopes (.5,.5) -> .7 ; then 3 quiet iterations
    assert rows[2][0] and abs(rows[2][2] - 0.7) < 1e-6
    assert [r[0] for r in rows[3:6]] == [False, False, True]
    assert abs(rows[5][2] - 1.4 * (0.5 + drift_after(3) / 3) / 2) < 1e-6


def test_first_event_without_forcing_uses_k_minus_minus_one(oracle_mod):
    # delta_init > 0, no forcing: first event when drift reaches delta_init, slope divides by k+1
    _, rows = scalar_run(oracle_mod, 6, thr_mode=1, horizon=1.0, delta_init=1.2, force_first=0)
    # nobody has sent: plain SGD, drift = 0.5 k  -> first event at k = 3 (1.5 >= 1.2)
    assert [r[0] for r in rows[:4]] == [False, False, False, True]
    assert abs(rows[3][2] - 1.5 / 4) < 1e-7


# --------------------------------------------------------------------------
# bookkeeping invariants (Section 5 error bound; Section 4 update of xhat)
# --------------------------------------------------------------------------
def run_and_check_invariants(oracle_mod, w, iters, **over):
    o = oracle_mod.Oracle.from_workload(w, **over)
    numel = w.layer_numel.astype(np.int64)
    off = np.concatenate([[0], np.cumsum(numel)])
    P, L = w.P, w.L
    delta_prev = o.tables()["delta"].copy()
    for k in range(iters):
        x_prev, xhat_prev = o.state("x"), o.state("xhat")
        o.step(k)
        d = o.decisions()
        tb = o.tables()
        xhat = o.state("xhat")
        ml, mr = o.state("mbox_l"), o.state("mbox_r")
        for r in range(P):
            for l in range(L):
                sl = slice(off[l], off[l + 1])
                diff = x_prev[r, sl].astype(np.float64) - xhat_prev[r, sl].astype(np.float64)
                nrm = math.sqrt(float(np.dot(diff, diff)))
                assert abs(d["norm"][r, l] - nrm) <= 1e-6 * nrm + 1e-30
                if d["fired"][r, l] == 0:
                    assert d["norm"][r, l] < d["delta_before"][r, l]           # error bound
                    assert np.array_equal(xhat[r, sl], xhat_prev[r, sl])
                    assert tb["delta"][r, l] == delta_prev[r, l]               # held between events
                elif d["fired"][r, l] == 1:
                    assert np.array_equal(xhat[r, sl], x_prev[r, sl])
                else:
                    idx, val = o.message(r, l)
                    K = oracle_mod.topk_count(numel[l], w.topk_ppm)
                    assert idx.size == K and np.all(np.diff(idx.astype(np.int64)) > 0)
                    assert np.array_equal(val, x_prev[r, sl][idx])
                    want = xhat_prev[r, sl].copy()
                    want[idx] = val
                    assert np.array_equal(xhat[r, sl], want)
                if d["fired"][r, l] or k == 0 and w.force_first:
                    assert d["fired"][r, l]
                # ring addressing: my right neighbour's left slot and my left
                # neighbour's right slot hold exactly what I last sent
                if tb["last_event_iter"][r, l] >= 0:
                    assert tb["valid_l"][(r + 1) % P, l] and tb["valid_r"][(r - 1) % P, l]
                    assert np.array_equal(ml[(r + 1) % P, sl], xhat[r, sl])
                    assert np.array_equal(mr[(r - 1) % P, sl], xhat[r, sl])
                else:
                    assert not tb["valid_l"][(r + 1) % P, l] and not tb["valid_r"][(r - 1) % P, l]
        delta_prev = tb["delta"].copy()
        assert np.isfinite(o.state("x")).all()
    return o


def small_workload(**kw):
    base = inputs.Workload("toy", 5, inputs.mlp((24, 10, 4)), 30, sigma0=0.02, decay=0.97)
    return base.scaled(**kw)


def test_invariants_fixed_threshold(oracle_mod):
    o = run_and_check_invariants(oracle_mod, small_workload(thr_mode=0, thr_fixed=4e-3), 30)
    t = o.totals()
    assert 5 * 4 <= t["events_total"] < 5 * 4 * 30      # some, not all
    assert t["index_words"] == 0 and t["bytes_sent"] == 8 * t["value_words"]


def test_invariants_adaptive(oracle_mod):
    o = run_and_check_invariants(oracle_mod, small_workload(), 30)
    t = o.totals()
    assert 5 * 4 * 2 <= t["events_total"] < 5 * 4 * 30   # k = 0 and k = 1 always fire (delta_init = 0)


def test_invariants_topk(oracle_mod):
    w = small_workload(topk_ppm=100_000)
    o = run_and_check_invariants(oracle_mod, w, 30)
    t, tb = o.totals(), o.tables()
    assert (tb["events_full"] == 1).all()                # a tensor's first event travels whole
    K = np.array([oracle_mod.topk_count(n, w.topk_ppm) for n in w.layer_numel])
    assert t["index_words"] == int((tb["events_topk"] * K[None, :]).sum())
    assert t["value_words"] == t["index_words"] + w.P * w.N
    # Section 7: a Top-K message is 2K% of a full one
    assert t["bytes_sent"] == 8 * (t["value_words"] + t["index_words"])


def test_forced_first_event_and_no_forcing(oracle_mod):
    w = small_workload(thr_mode=0, thr_fixed=10.0)
    o = oracle_mod.Oracle.from_workload(w)
    o.step(0)
    assert o.decisions()["fired"].all() and o.tables()["valid_l"].all() and o.tables()["valid_r"].all()
    o.step(1)
    assert not o.decisions()["fired"].any()
    o = oracle_mod.Oracle.from_workload(w, force_first=0)
    o.step(0)
    assert not o.decisions()["fired"].any()


def test_nan_drift_never_fires_and_is_counted(oracle_mod):
    numel = [4, 4]
    x0 = np.ones((3, 8), np.float32)
    o = oracle_mod.Oracle(x0, np.array(numel, np.uint64), None, thr_mode=0, thr_fixed=0.5,
                          force_first=0, grad_mode=1, lr=1.0, momentum=0.0)
    g = np.zeros((3, 8), np.float32)
    g[1, 0] = np.nan
    o.step(0, grad=g)
    o.step(1, grad=np.zeros_like(g))
    d = o.decisions()
    assert math.isnan(d["norm"][1, 0]) and d["fired"][1, 0] == 0
    assert o.totals()["nonfinite_norms"] == 1
    # +inf drift against +inf threshold fires (IEEE >=)
    o = oracle_mod.Oracle(x0, np.array(numel, np.uint64), None, thr_mode=0, thr_fixed=INF,
                          force_first=0, grad_mode=1, lr=1.0, momentum=0.0)
    g[1, 0] = np.inf
    o.step(0, grad=g)
    o.step(1, grad=np.zeros_like(g))
    assert o.decisions()["fired"][1, 0] == 1


# --------------------------------------------------------------------------
# Top-K selection (Section 7) against brute force
# --------------------------------------------------------------------------
def brute_topk(keys, K):
    order = sorted(range(len(keys)), key=lambda i: (-int(keys[i]), i))
    return np.array(sorted(order[:K]), np.uint32)


def test_topk_select_bruteforce(oracle_mod):
    rng = np.random.default_rng(0)
    for n in [1, 2, 5, 64, 257, 1000, 4096]:
        for K in sorted({1, max(1, n // 100), max(1, n // 10), n // 2 + 1, n}):
            for hi in (3, 50, 2**31):          # many ties ... almost none
                keys = rng.integers(0, hi, n, dtype=np.uint64).astype(np.uint32)
                assert np.array_equal(oracle_mod.topk_select(keys, K), brute_topk(keys, K))
    keys = np.full(100, 7, np.uint32)
    assert np.array_equal(oracle_mod.topk_select(keys, 13), np.arange(13, dtype=np.uint32))


def test_topk_count_rounding(oracle_mod):
    assert oracle_mod.topk_count(10, 100_000) == 1
    assert oracle_mod.topk_count(11, 100_000) == 2        # ceil
    assert oracle_mod.topk_count(3, 10_000) == 1          # never zero
    assert oracle_mod.topk_count(2_359_296, 100_000) == 235_930
    assert oracle_mod.topk_count(2_359_296, 10_000) == 23_593
    assert oracle_mod.topk_count(77, 1_000_000) == 77


def test_topk_ranks_by_drift_magnitude_with_index_tiebreak(oracle_mod):
    numel = [10]
    P = 3
    x0 = np.full((P, 10), 5.0, np.float32)      # non-zero, so |x - xhat|, |x + xhat| and |x| rank differently
    o = oracle_mod.Oracle(x0, np.array(numel, np.uint64), None, thr_mode=0, thr_fixed=0.0,
                          topk_ppm=300_000, grad_mode=1, lr=1.0, momentum=0.0)
    zero = np.zeros((P, 10), np.float32)
    o.step(0, grad=zero)                    # first event: whole tensor
    assert (o.decisions()["fired"] == 1).all()
    g = np.zeros((P, 10), np.float32)
    g[0] = [0.1, -3, 2, 2, -2, 0, 0.5, 2, -0.2, 1]       # drift after the step = -g
    o.step(1, grad=g)                       # step 1 sends zero drift: ties -> indices 0,1,2
    assert np.array_equal(o.message(0, 0)[0], [0, 1, 2])
    o.step(2, grad=zero)
    idx, val = o.message(0, 0)
    assert np.array_equal(idx, [1, 2, 3])   # |-3| then the lowest two indices among |2| ties
    # key option 1 ranks by |x| instead
    o1 = oracle_mod.Oracle(np.zeros((P, 10), np.float32) + np.arange(10, dtype=np.float32)[None, :], np.array(numel, np.uint64),
                           None, thr_mode=0, thr_fixed=0.0, topk_ppm=300_000, topk_key=1,
                           grad_mode=1, lr=1.0, momentum=0.0)
    o1.step(0, grad=zero)
    o1.step(1, grad=zero)
    assert np.array_equal(o1.message(0, 0)[0], [7, 8, 9])


def test_topk_everything_equals_full_send(oracle_mod):
    w = small_workload()
    a = oracle_mod.Oracle.from_workload(w)
    b = oracle_mod.Oracle.from_workload(w, topk_ppm=1_000_000)
    for k in range(25):
        a.step(k)
        b.step(k)
        assert np.array_equal(a.decisions()["fired"] > 0, b.decisions()["fired"] > 0)
    for name in ("x", "xhat", "mbox_l", "mbox_r", "vel"):
        assert np.array_equal(a.state(name), b.state(name))


def test_xhat_reset_reading_of_a_topk_event(oracle_mod):
    """xhat_reset = 1: a Top-K event resets the whole tensor's xhat to x (Section 4's
    per-tensor xhat), while the neighbours' copies change only at the sent indices.
    Checked against the states observed before each step: winners by brute force on
    |x - xhat|, xhat == x for the whole tensor, untouched mailbox entries keep their values."""
    w = small_workload(topk_ppm=200_000)
    o = oracle_mod.Oracle.from_workload(w, xhat_reset=1)
    ref = oracle_mod.Oracle.from_workload(w)              # default reading, same inputs
    numel = w.layer_numel.astype(np.int64)
    off = np.concatenate([[0], np.cumsum(numel)])
    P, L = w.P, w.L
    seen_topk = differs = 0
    for k in range(30):
        x_prev, xhat_prev = o.state("x"), o.state("xhat")
        ml_prev, mr_prev = o.state("mbox_l"), o.state("mbox_r")
        o.step(k)
        ref.step(k)
        d = o.decisions()
        xhat, ml, mr = o.state("xhat"), o.state("mbox_l"), o.state("mbox_r")
        for r in range(P):
            for l in range(L):
                sl = slice(off[l], off[l + 1])
                if d["fired"][r, l] == 0:
                    assert np.array_equal(xhat[r, sl], xhat_prev[r, sl])
                    continue
                assert np.array_equal(xhat[r, sl], x_prev[r, sl])           # whole tensor, either kind of event
                if d["fired"][r, l] != 2:
                    continue
                seen_topk += 1
                idx, val = o.message(r, l)
                keys = np.abs(x_prev[r, sl] - xhat_prev[r, sl]).astype(np.float32).view(np.uint32)
                K = oracle_mod.topk_count(numel[l], w.topk_ppm)
                assert np.array_equal(idx, brute_topk(keys, K))
                assert np.array_equal(val, x_prev[r, sl][idx])
                for box, box_prev, nb in ((ml, ml_prev, (r + 1) % P), (mr, mr_prev, (r - 1) % P)):
                    want = box_prev[nb, sl].copy()
                    want[idx] = val
                    assert np.array_equal(box[nb, sl], want, equal_nan=True)
    assert seen_topk > 50
    # the reading matters: the two runs part ways (under the default one unsent drift carries over)
    assert not np.array_equal(o.state("xhat"), ref.state("xhat"))
    assert not np.array_equal(o.state("x"), ref.state("x"))
    t = o.totals()
    assert t["index_words"] > 0 and t["bytes_sent"] == 8 * (t["value_words"] + t["index_words"])


def test_xhat_reset_with_everything_sent_is_the_whole_send(oracle_mod):
    w = small_workload()
    a = oracle_mod.Oracle.from_workload(w)
    b = oracle_mod.Oracle.from_workload(w, topk_ppm=1_000_000, xhat_reset=1)
    for k in range(25):
        a.step(k)
        b.step(k)
    for name in ("x", "xhat", "mbox_l", "mbox_r", "vel"):
        assert np.array_equal(a.state(name), b.state(name))


# --------------------------------------------------------------------------
# determinism, overrides, final average
# --------------------------------------------------------------------------
def test_determinism_and_seed_sensitivity(oracle_mod):
    w = small_workload(topk_ppm=200_000)
    runs = []
    for seed in (5, 5, 6):
        o = oracle_mod.Oracle.from_workload(w.scaled(seed=seed), x0=inputs.replicate(w.x0(), w.P))
        for k in range(15):
            o.step(k)
        runs.append(o.state("x"))
    assert np.array_equal(runs[0], runs[1])
    assert not np.array_equal(runs[0], runs[2])


def test_override_only_on_flagged_near_ties(oracle_mod):
    # the scalar toy has a genuine tie d == delta at every k >= 2 (h = 1)
    P = 3
    mk = lambda: oracle_mod.Oracle(np.zeros((P, 1), np.float32), np.array([1], np.uint64), None,
                                   lr=0.5, momentum=0.0, grad_mode=1, thr_mode=1)
    g = np.ones((P, 1), np.float32)
    o = mk()
    for k in range(2):
        o.step(k, grad=g)
    o.step(2, grad=g, override=np.array([0, -1, -1], np.int8))
    d = o.decisions()
    assert d["near_tie"].all() and list(d["fired"][:, 0]) == [0, 1, 1]
    # an override where nothing is near a tie is ignored
    o = mk()
    o.step(0, grad=g)
    o.step(1, grad=g, override=np.zeros(3, np.int8))
    assert o.decisions()["fired"].all() and not o.decisions()["near_tie"].any()


def test_final_average(oracle_mod):
    o, x0 = make(oracle_mod, [6, 3], 4, thr_mode=0, thr_fixed=0.0, grad_mode=1)
    np.testing.assert_allclose(o.average(), x0.astype(np.float64).mean(0), rtol=1e-6)


def test_rejects_bad_configurations(oracle_mod):
    with pytest.raises(ValueError):
        oracle_mod.Oracle(np.zeros((2, 4), np.float32), np.array([4], np.uint64))   # ring needs >= 3
    o, _ = make(oracle_mod, [4], 3, grad_mode=1)
    with pytest.raises(RuntimeError):
        o.step(0)                          # buffer mode without a buffer
    o.step(0, grad=np.zeros((3, 4), np.float32))
    with pytest.raises(RuntimeError):
        o.step(0, grad=np.zeros((3, 4), np.float32))   # iterations must increase


# --------------------------------------------------------------------------
# the other reading of Section 4's wording: the norm itself has to change
# --------------------------------------------------------------------------
def test_norm_difference_trigger_ignores_rotations(oracle_mod):
    """A tensor that turns from (1,0) to (0,1) has moved by sqrt(2) but its norm has not
    changed: the drift-norm trigger fires, the norm-difference trigger stays silent until
    the length changes."""
    P = 3
    x0 = np.tile(np.array([[1.0, 0.0]], np.float32), (P, 1))
    mk = lambda kind: oracle_mod.Oracle(x0, np.array([2], np.uint64), None, lr=1.0, momentum=0.0,
                                        thr_mode=0, thr_fixed=0.5, grad_mode=1, trigger_kind=kind)
    g0 = np.tile(np.array([[1.0, -1.0]], np.float32), (P, 1))       # (1,0) -> (0,1)
    zero = np.zeros_like(g0)
    a, b = mk(0), mk(1)
    for o in (a, b):
        o.step(0, grad=g0)
        assert o.decisions()["fired"].all()                        # forced first event
        assert np.array_equal(o.state("x"), np.tile(np.array([[0.0, 1.0]], np.float32), (P, 1)))
        o.step(1, grad=zero)
    da, db = a.decisions(), b.decisions()
    assert da["fired"].all() and abs(da["norm"][0, 0] - math.sqrt(2)) < 1e-6
    assert not db["fired"].any() and db["norm"][0, 0] == 0.0
    # b: x = (0,1) + 2/3 ((1,0) - (0,1)) = (2/3, 1/3); push it out to length 2
    x = b.state("x")[0].astype(np.float64)
    np.testing.assert_allclose(x, [2 / 3, 1 / 3], atol=1e-6)
    b.step(2, grad=zero)            # |x| = sqrt(5)/3 = 0.745: changed by 0.255 < 0.5, still silent
    d = b.decisions()
    assert not d["fired"].any() and abs(d["norm"][0, 0] - (1 - math.sqrt(5) / 3)) < 1e-6
    x = b.state("x")[0].astype(np.float64)
    g = np.tile((x + 2 / 3 * (np.array([1.0, 0.0]) - x) - np.array([2.0, 0.0]))[None, :], (P, 1)).astype(np.float32)
    b.step(3, grad=g)               # lands on (2, 0)
    b.step(4, grad=zero)
    d = b.decisions()
    assert d["fired"].all() and abs(d["norm"][0, 0] - 1.0) < 1e-5   # | 2 - 1 |


def test_norm_difference_trigger_adaptive_and_topk_invariants(oracle_mod):
    w = small_workload(topk_ppm=200_000)
    o = oracle_mod.Oracle.from_workload(w, trigger_kind=1)
    numel = w.layer_numel.astype(np.int64)
    off = np.concatenate([[0], np.cumsum(numel)])
    for k in range(25):
        x_prev, h_prev = o.state("x"), o.state("xhat")
        o.step(k)
        d = o.decisions()
        for r in range(w.P):
            for l in range(w.L):
                sl = slice(off[l], off[l + 1])
                nx = np.float32(math.sqrt(float(np.dot(x_prev[r, sl].astype(np.float64), x_prev[r, sl].astype(np.float64)))))
                nh = np.float32(math.sqrt(float(np.dot(h_prev[r, sl].astype(np.float64), h_prev[r, sl].astype(np.float64)))))
                assert abs(d["norm"][r, l] - abs(float(nx) - float(nh))) <= 2e-6 * float(nx)
                if d["fired"][r, l] == 0:
                    assert d["norm"][r, l] < d["delta_before"][r, l]
    t = o.totals()
    assert w.P * w.L * 2 <= t["events_total"] < w.P * w.L * 25


# --------------------------------------------------------------------------
# delayed delivery: what is sent in iteration k is averaged in from iteration k + 1
# --------------------------------------------------------------------------
@pytest.mark.parametrize("P", [3, 5])
def test_delayed_delivery_is_dpsgd_with_one_step_old_neighbours(oracle_mod, P):
    numel = [6, 17]
    n = sum(numel)
    lr, mu = 0.05, 0.9
    o, x0 = make(oracle_mod, numel, P, thr_mode=0, thr_fixed=0.0, lr=lr, momentum=mu, grad_mode=1,
                 delivery_delay=1)
    W = ring_matrix(P)
    Wn = W - np.eye(P) / 3.0               # the neighbours' part of the mixing matrix
    X = x0.astype(np.float64).T
    X_old = None
    V = np.zeros_like(X)
    for k in range(20):
        g = inputs.random_grads(P, n, 300 + k, 0.1)
        o.step(k, grad=g)
        V = mu * V + g.astype(np.float64).T
        if X_old is None:
            X_new = X - lr * V             # nothing has arrived yet: a plain local step
        else:
            X_new = X / 3.0 + X_old @ Wn - lr * V
        X_old, X = X, X_new
        np.testing.assert_allclose(o.state("x").T, X, rtol=0, atol=2e-6 * np.abs(X).max())
    tb = o.tables()
    assert tb["valid_l"].all() and tb["valid_r"].all()


def test_delayed_delivery_topk_keeps_the_ring_invariant(oracle_mod):
    w = small_workload(topk_ppm=200_000)
    o = oracle_mod.Oracle.from_workload(w, delivery_delay=1)
    numel = w.layer_numel.astype(np.int64)
    off = np.concatenate([[0], np.cumsum(numel)])
    for k in range(20):
        o.step(k)
        xhat, ml, mr, tb = o.state("xhat"), o.state("mbox_l"), o.state("mbox_r"), o.tables()
        for r in range(w.P):
            for l in range(w.L):
                sl = slice(off[l], off[l + 1])
                if tb["last_event_iter"][r, l] >= 0:      # delivered by the end of the iteration
                    assert np.array_equal(ml[(r + 1) % w.P, sl], xhat[r, sl])
                    assert np.array_equal(mr[(r - 1) % w.P, sl], xhat[r, sl])
    a = oracle_mod.Oracle.from_workload(w)
    for k in range(20):
        a.step(k)
    assert not np.array_equal(a.state("x"), o.state("x"))     # the delay does change the run
