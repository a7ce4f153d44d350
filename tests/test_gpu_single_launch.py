"""Rings that take ONE kernel launch per iteration: cache-resident, whole-tensor sends, norms
accumulated by the update pass, no tensor above 128 sweeps.  Their update pass runs the trigger
tests itself (every workgroup the three it depends on), on arrays that the same launch does not
write.  Checked here: the path is the one that runs (no samples of the trigger phase), it equals
the oracle step by step in every mode it serves, it hands over to the other launch sequences
and back (evg_step_next, checkpoints at odd and even step counts), and rings that do not
qualify keep the separate trigger kernel."""
import numpy as np
import pytest

from paper_2103_07454_amd import inputs

pytestmark = pytest.mark.gpu

ARENAS = ("x", "xhat", "vel", "mbox_l", "mbox_r")
TENSORS = [inputs.TensorSpec("w0", (4097,), 16, "weight"), inputs.TensorSpec("b0", (1,), 16, "bias"),
           inputs.TensorSpec("w1", (9000,), 32, "weight"), inputs.TensorSpec("b1", (7,), 32, "bias"),
           inputs.TensorSpec("w2", (1023,), 8, "weight"), inputs.TensorSpec("w3", (1024,), 8, "weight"),
           inputs.TensorSpec("w4", (100_353,), 64, "weight"), inputs.TensorSpec("b4", (2,), 64, "bias")]


@pytest.fixture(scope="module")
def evg():
    from paper_2103_07454_amd import evg as m
    m.lib()
    return m


def workload(P=5, tensors=TENSORS, iters=30, **kw):
    base = inputs.Workload("single_launch", P, tensors, iters, sigma0=0.05, fan_in_scaling=1, decay=0.98,
                           spike_prob=0.15, spike_gain=4.0, seed=4242)
    return base.scaled(**kw)


def trigger_launches(ring):
    return ring.timing_read()["trigger"][1]


def same(a, b):
    da, db = a.decisions(), b.decisions()
    for key in ("fired", "near_tie", "norm", "delta_before"):
        assert np.array_equal(da[key], db[key]), key
    for name in ARENAS:
        assert np.array_equal(a.state(name), b.state(name), equal_nan=True), name
    sa, sb = a.stats(arrays=True), b.stats(arrays=True)
    for key in sa:
        if key != "library_bytes":
            assert np.array_equal(sa[key], sb[key]), key


# mode -> (workload fields, options given to both sides)
MODES = dict(
    adaptive=(dict(), dict()),
    fixed=(dict(thr_mode=inputs.THR_FIXED, thr_fixed=6e-2), dict()),
    history3=(dict(horizon=1.3), dict(hist_len=3)),
    student=(dict(dist=inputs.DIST_STUDENT_T3), dict()),
    plain_sgd=(dict(momentum=0.0), dict()),
    three_workers=(dict(P=3), dict()),
    no_forced_first_event=(dict(force_first=0, delta_init=0.02), dict()),
)


@pytest.mark.parametrize("mode", list(MODES))
def test_single_launch_steps_equal_the_oracle(evg, oracle_mod, mode):
    from helpers import lockstep
    fields, over = MODES[mode]
    w = workload(**fields)
    x0 = inputs.replicate(w.x0(), w.P)
    ring = evg.Ring.from_workload(w, x0, mailbox_fill=float("nan"), **over)
    ring.timing(True)
    orc = oracle_mod.Oracle.from_workload(w, x0, **over)
    rep = lockstep(ring, orc, w.iters, sample_messages=0)
    assert all(rep["bitwise"].values()), rep
    st = ring.stats()
    assert 0 < st["events_total"] < st["regular_events"]
    t = ring.timing_read()
    assert t["trigger"][1] == 0 and t["send_full"][1] == 0 and t["update"][1] == w.iters


@pytest.mark.parametrize("separate_norm", [False, True])
def test_norm_difference_trigger_in_a_single_launch(evg, oracle_mod, separate_norm):
    from helpers import lockstep
    w = workload()
    x0 = inputs.replicate(w.x0(), w.P)
    over = dict(trigger_kind=1)
    gpu = dict(norm_mode=evg.NORM_SEPARATE) if separate_norm else {}
    ring = evg.Ring.from_workload(w, x0, mailbox_fill=float("nan"), **over, **gpu)
    ring.timing(True)
    orc = oracle_mod.Oracle.from_workload(w, x0, **over)
    rep = lockstep(ring, orc, w.iters, sample_messages=0, norm_abs_of_x=2.5e-7)
    assert all(rep["bitwise"].values()), rep
    # a separate norm pass must come before the tests: such rings keep the trigger kernel
    assert trigger_launches(ring) == (w.iters if separate_norm else 0)


def test_gradients_from_a_buffer_in_a_single_launch(evg, oracle_mod):
    import torch
    from helpers import lockstep
    w = workload(iters=12)
    x0 = inputs.replicate(w.x0(), w.P)
    ring = evg.Ring.from_workload(w, x0, mailbox_fill=float("nan"), grad_mode=1)
    ring.timing(True)
    orc = oracle_mod.Oracle.from_workload(w, x0, grad_mode=1)
    keep = []

    def host(k):
        return inputs.random_grads(w.P, w.N, 700 + k, 0.02)

    def dev(k):
        keep.append(torch.from_numpy(ring.layout.pad(host(k))).cuda())
        return keep[-1]

    rep = lockstep(ring, orc, w.iters, grads=host, gpu_grads=dev, sample_messages=0)
    assert all(rep["bitwise"].values()), rep
    assert trigger_launches(ring) == 0


def test_rings_that_do_not_qualify_keep_the_trigger_kernel(evg, oracle_mod):
    from helpers import lockstep
    # one tensor of 129 sweeps; streaming accesses; Top-K; delayed delivery
    long_tensor = TENSORS[:2] + [inputs.TensorSpec("w9", (128 * 1024 + 1,), 64, "weight")]
    cases = [(workload(tensors=long_tensor, iters=8), {}, {}),
             (workload(iters=8), {}, dict(access_mode=evg.ACCESS_STREAM)),
             (workload(iters=8, topk_ppm=100_000), {}, {}),
             (workload(iters=8), dict(delivery_delay=1), {})]
    for w, over, gpu in cases:
        x0 = inputs.replicate(w.x0(), w.P)
        ring = evg.Ring.from_workload(w, x0, mailbox_fill=float("nan"), **over, **gpu)
        ring.timing(True)
        orc = oracle_mod.Oracle.from_workload(w, x0, **over)
        rep = lockstep(ring, orc, w.iters, sample_messages=8)
        assert all(rep["bitwise"].values()), rep
        assert trigger_launches(ring) == w.iters


def test_hand_over_to_the_replayable_step_and_back(evg):
    """evg_step (single launch) and evg_step_next (trigger kernel first) continue each other; after
    the first evg_step_next every step of that ring takes the trigger kernel."""
    w = workload()
    a = evg.Ring.from_workload(w)                                         # single launch throughout
    b = evg.Ring.from_workload(w)                                         # mixes
    c = evg.Ring.from_workload(w, access_mode=evg.ACCESS_STREAM)          # never single launch
    for r in (a, b, c):
        r.timing(True)
    for k in range(5):                      # an odd number of steps: the second set of arrays is current
        for r in (a, b, c):
            r.step(k)
    same(a, b); same(a, c)
    for k in range(5, 8):
        a.step(k); c.step(k)
        b.step_next()
    same(a, b); same(a, c)
    for k in range(8, 14):
        for r in (a, b, c):
            r.step(k)
        same(a, b)
    same(a, c)
    assert trigger_launches(a) == 0 and trigger_launches(c) == 14
    assert trigger_launches(b) == 6         # evg_step after the first evg_step_next (which is not timed)


@pytest.mark.parametrize("steps_before", [5, 6])
@pytest.mark.parametrize("norm_diff", [0, 1])
def test_checkpoints_of_single_launch_rings(evg, steps_before, norm_diff):
    """The blob holds whichever set of arrays is current (odd / even step counts), and a ring of the
    other launch sequence continues from it bit for bit, and the other way round."""
    w = workload(horizon=1.2)
    over = dict(trigger_kind=norm_diff, hist_len=2)
    a = evg.Ring.from_workload(w, **over)
    s = evg.Ring.from_workload(w, access_mode=evg.ACCESS_STREAM, **over)
    for k in range(steps_before):
        a.step(k); s.step(k)
    blob_a, blob_s = a.export_state(), s.export_state()
    a2 = evg.Ring.from_workload(w, **over)                                # single launch, from the streaming ring's blob
    s2 = evg.Ring.from_workload(w, access_mode=evg.ACCESS_STREAM, **over)  # and the reverse
    a2.import_state(blob_s)
    s2.import_state(blob_a)
    for r in (a, a2, s2):
        r.timing(True)
    for k in range(steps_before, steps_before + 9):
        for r in (a, s, a2, s2):
            r.step(k)
        same(a, s); same(a, a2); same(a, s2)
    assert trigger_launches(a) == 0 and trigger_launches(a2) == 0 and trigger_launches(s2) == 9
