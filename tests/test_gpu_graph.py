"""evg_step_next: the step whose iteration lives in device memory, eager and replayed
from a captured HIP graph.  Every replay is compared with a ring stepped by evg_step."""
import numpy as np
import pytest

from paper_2103_07454_amd import inputs

pytestmark = pytest.mark.gpu

ARENAS = ("x", "xhat", "vel", "mbox_l", "mbox_r")
TENSORS = [inputs.TensorSpec("w0", (4097,), 16, "weight"), inputs.TensorSpec("b0", (1,), 16, "bias"),
           inputs.TensorSpec("w1", (9000,), 32, "weight"), inputs.TensorSpec("w2", (20481,), 64, "weight"),
           inputs.TensorSpec("b2", (3,), 64, "bias")]


@pytest.fixture(scope="module")
def evg():
    from paper_2103_07454_amd import evg as m
    m.lib()
    return m


def workload(**kw):
    base = inputs.Workload("graph", 5, TENSORS, 40, sigma0=0.05, fan_in_scaling=1, decay=0.97,
                           spike_prob=0.2, spike_gain=4.0, seed=31)
    return base.scaled(**kw)


def same(a, b):
    da, db = a.decisions(), b.decisions()
    assert np.array_equal(da["fired"], db["fired"]) and np.array_equal(da["norm"], db["norm"])
    for name in ARENAS:
        assert np.array_equal(a.state(name), b.state(name), equal_nan=True), name
    sa, sb = a.stats(arrays=True), b.stats(arrays=True)
    for key in sa:
        assert np.array_equal(sa[key], sb[key]), key


@pytest.mark.parametrize("topk", [0, 100_000])
def test_step_next_is_the_next_iteration(evg, topk):
    w = workload(topk_ppm=topk)
    a = evg.Ring.from_workload(w)
    b = evg.Ring.from_workload(w)
    for k in range(6):
        a.step(k)
        b.step_next()
    same(a, b)
    # the two calls mix: evg_step continues after what evg_step_next reached, and refuses to go back
    with pytest.raises(evg.EvgError) as e:
        b.step(5)
    assert e.value.status == 5
    a.step(6); b.step(6)
    a.step(9); b.step(9)                 # a gap in the numbering
    a.step(10); b.step_next()
    same(a, b)
    assert b.stats()["iters"] == 9
    # and the state blob carries the device's iteration along
    ck = b.export_state()
    c = evg.Ring.from_workload(w)
    c.import_state(ck)
    a.step(11); c.step_next()
    same(a, c)


@pytest.mark.parametrize("topk,buffer", [(0, False), (100_000, False), (100_000, True)])
def test_captured_step_replays_as_successive_iterations(evg, topk, buffer):
    import torch
    w = workload(topk_ppm=topk)
    over = dict(grad_mode=evg.GRAD_BUFFER) if buffer else {}
    ref = evg.Ring.from_workload(w, **over)
    g = None
    if buffer:       # the captured graph keeps reading this one array
        g = torch.from_numpy(ref.layout.pad(inputs.random_grads(w.P, w.N, 8, 0.02))).cuda()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        ring = evg.Ring.from_workload(w, stream=s, **over)
        ring.step_next(g)                     # iterations 0 and 1, eagerly
        ring.step_next(g)
    s.synchronize()
    ref.step(0, g)
    ref.step(1, g)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        ring.step_next(g)                     # recorded, not run
    same(ref, ring)                           # the capture itself changed nothing
    junk = torch.zeros(1 << 20, device="cuda")
    for k in range(2, 12):
        graph.replay()
        ref.step(k, g)
        junk.add_(1.0)                        # eager work of the program's own between replays
        torch.cuda.synchronize()
        same(ref, ring)
    assert ring.stats()["iters"] == 12 and float(junk[0]) == 10.0
    ring.step(12, g); ref.step(12, g)         # back to the eager call
    same(ref, ring)
