"""GPU parity over seeded random configurations: ring size, tensor sizes, thresholds,
send mode, Top-K share and key, history length, trigger kind, delivery, gradient
distribution, chunking and access mode are all drawn at random (fixed seeds), and every
run is stepped in lock-step with the oracle."""
import numpy as np
import pytest

from paper_2103_07454_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def evg():
    from paper_2103_07454_amd import evg as m
    m.lib()
    return m


def draw(rng):
    P = int(rng.integers(3, 10))
    L = int(rng.integers(1, 9))
    sizes = []
    for _ in range(L):
        kind = rng.integers(4)
        if kind == 0:
            sizes.append(int(rng.integers(1, 9)))
        elif kind == 1:
            sizes.append(int(rng.integers(9, 1100)))
        elif kind == 2:
            sizes.append(int(rng.integers(1100, 9000)))
        else:
            sizes.append(int(rng.integers(9000, 40000)))
    tensors = [inputs.TensorSpec(f"t{i}", (n,), int(rng.integers(1, 64)), "weight") for i, n in enumerate(sizes)]
    topk = bool(rng.integers(2))
    adaptive = bool(rng.integers(3))          # two in three
    w = inputs.Workload(
        "random", P, tensors, 14, lr=float(rng.choice([0.01, 0.05, 0.2])), momentum=float(rng.choice([0.0, 0.5, 0.9])),
        thr_mode=inputs.THR_ADAPTIVE if adaptive else inputs.THR_FIXED,
        thr_fixed=float(rng.choice([0.0, 1e-3, 2e-2, 0.3])), horizon=float(rng.choice([0.7, 1.0, 1.5])),
        delta_init=float(rng.choice([0.0, 0.0, 0.05])), force_first=int(rng.integers(2)),
        topk_ppm=int(rng.choice([1, 10_000, 100_000, 333_333, 900_000])) if topk else 0,
        dist=int(rng.integers(2)), sigma0=float(rng.choice([0.0, 0.01, 0.1])), fan_in_scaling=int(rng.integers(2)),
        decay=float(rng.choice([1.0, 0.97, 0.8])), spike_prob=float(rng.choice([0.0, 0.3])), spike_gain=4.0,
        seed=int(rng.integers(1 << 40)))
    both = dict(hist_len=int(rng.choice([1, 1, 2, 5])), trigger_kind=int(rng.integers(2)),
                topk_key=int(rng.integers(2)) if topk else 0)
    delay = int(rng.integers(3) == 0)
    both["delivery_delay"] = delay
    both["xhat_reset"] = int(topk and not delay and rng.integers(3) == 0)
    gpu = dict(chunk_elems=int(rng.choice([1024, 2048, 4096, 8192])), norm_mode=int(rng.integers(4) == 0),
               access_mode=int(rng.integers(3)))
    distinct = bool(rng.integers(2))
    return w, both, gpu, distinct


@pytest.mark.parametrize("case", range(120))
def test_random_configuration(evg, oracle_mod, case):
    from helpers import lockstep
    rng = np.random.default_rng(7_000 + case)
    w, both, gpu, distinct = draw(rng)
    x0 = inputs.distinct_params(w.N, w.P, 11 + case, 0.1) if distinct else inputs.replicate(w.x0(), w.P)
    tag = f"P={w.P} sizes={[int(n) for n in w.layer_numel]} topk={w.topk_ppm} thr={w.thr_mode}/{w.thr_fixed} " \
          f"{both} {gpu} dist={w.dist}"
    print("\n[random]", case, tag, flush=True)
    ring = evg.Ring.from_workload(w, x0, mailbox_fill=float("nan"), **both, **gpu)
    orc = oracle_mod.Oracle.from_workload(w, x0, **both)
    # the norm-difference trigger subtracts two large norms: decisions still must agree, norms only loosely
    rep = lockstep(ring, orc, w.iters, sample_messages=16, norm_rtol=None if both["trigger_kind"] else 2e-7,
                   norm_abs_of_x=2.5e-7 if both["trigger_kind"] else None)
    assert rep["rel"]["x"] <= 1e-5, tag
    if not both["trigger_kind"]:
        assert all(rep["bitwise"].values()), tag
    ring.close()
