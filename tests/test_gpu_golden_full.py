"""Configurations 3, 4 and 5 at FULL size for their FULL iteration counts on the GPU, checked
after every iteration against the CPU oracle's record of the same run
(tests/golden/cfgN_full.npz, written by tests/golden/make_goldens.py, which calls only the
oracle):

  * every trigger decision (0 / whole / Top-K) of every (worker, tensor, iteration): exact;
    a difference is tolerated nowhere -- where both sides flag a near tie the message says how
    to regenerate the record with the HIP path's decision (the parity rule's only licence);
  * near-tie flags: exact; norms and thresholds: relative 2e-7 / 4e-7 (summation order);
  * every Top-K message through its two fingerprints (index set; indices + values): exact;
  * running event / word / near-tie totals: exact;
  * every 10 iterations and at the end, each of the five arrays per (worker, tensor): the
    position-weighted sum of its bit patterns (exact: the arrays are bit-identical), its
    float64 sum, its max |v|, and sampled values within 1e-5 of the largest magnitude;
  * the per-(worker, tensor) tables after the last iteration.
"""
import os

import numpy as np
import pytest

from paper_2103_07454_amd import inputs

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
ARRAYS = ("x", "xhat", "vel", "mbox_l", "mbox_r")
REL_TOL = 1e-5
WEIGHT_MUL = 0x9E3779B97F4A7C15 - (1 << 64)     # the multiplier as a two's-complement int64


@pytest.fixture
def say(capsys):
    def emit(msg):
        with capsys.disabled():
            print(msg, flush=True)
    return emit


@pytest.fixture(scope="module")
def evg():
    from paper_2103_07454_amd import evg as m
    m.lib()
    return m


class GpuDigest:
    """The fingerprints of make_goldens.py, recomputed with torch on the device arrays."""

    def __init__(self, ring, numel):
        import torch
        self.torch, self.ring = torch, ring
        self.numel = [int(n) for n in numel]
        self.off = [int(o) for o in ring.layout.offsets]
        self.weights = []
        for n in self.numel:
            j = torch.arange(1, n + 1, dtype=torch.int64, device=ring.device)
            self.weights.append((j * WEIGHT_MUL) | 1)
        self.index = torch.from_numpy(ring.layout.index).to(ring.device)

    def fingerprint(self, name):
        torch = self.torch
        a = getattr(self.ring, name)
        P, L = a.shape[0], len(self.numel)
        bits = torch.empty((P, L), dtype=torch.int64, device=a.device)
        sums = torch.empty((P, L), dtype=torch.float64, device=a.device)
        maxabs = torch.empty((P, L), dtype=torch.float32, device=a.device)
        u = a.view(torch.int32)
        for l, (o, n) in enumerate(zip(self.off, self.numel)):
            sl = slice(o, o + n)
            v = u[:, sl].to(torch.int64) & 0xFFFFFFFF
            bits[:, l] = (v * self.weights[l]).sum(dim=1)
            sums[:, l] = a[:, sl].sum(dim=1, dtype=torch.float64)
            maxabs[:, l] = a[:, sl].abs().amax(dim=1)
        return (bits.cpu().numpy().view(np.uint64), sums.cpu().numpy(), maxabs.cpu().numpy())

    def sample(self, name, flat_index):
        """Values at positions of the unpadded [P, N] layout."""
        torch = self.torch
        N = int(self.index.numel())
        idx = torch.from_numpy(np.asarray(flat_index, np.int64)).to(self.ring.device)
        pos = (idx // N) * self.ring.layout.npad + self.index[idx % N]
        return getattr(self.ring, name).reshape(-1)[pos].cpu().numpy()


def compare_digest(dg, g, d, k, say, tag, final):
    for name in ARRAYS:
        bits, sums, maxabs = dg.fingerprint(name)
        want_bits = g[f"dg_{name}_bits"][d]
        got = dg.sample(name, g["sample_index"])
        want = g[f"dg_{name}_sample"][d]
        scale = float(g[f"dg_{name}_maxabs"][d].max())
        err = float(np.abs(got.astype(np.float64) - want.astype(np.float64)).max()) / scale
        assert err <= REL_TOL, f"{tag} iteration {k}: {name} differs by {err:.3g} of its largest magnitude"
        np.testing.assert_allclose(sums, g[f"dg_{name}_sum"][d], rtol=1e-9,
                                   atol=1e-9 * scale * max(dg.numel),
                                   err_msg=f"{tag} iteration {k}: float64 sums of {name}")
        assert np.array_equal(maxabs, g[f"dg_{name}_maxabs"][d]), f"{tag} iteration {k}: max |{name}|"
        bad = np.argwhere(bits != want_bits)
        assert bad.size == 0, (f"{tag} iteration {k}: {name} is not bit-identical to the oracle's for "
                               f"(worker, tensor) {bad[:5].tolist()} (sampled values agree to {err:.3g})")
        if final:
            got = dg.sample(name, g["final_sample_index"])
            assert np.array_equal(got, g[f"final_{name}_sample"]), f"{tag}: final sample of {name}"
    say(f"{tag} iteration {k + 1}: all five arrays bit-identical to the oracle's record")


@pytest.mark.timeout(900)
@pytest.mark.parametrize("i", [3, 4, 5])
def test_full_size_full_length_run_matches_the_oracle_record(evg, say, i):
    path = os.path.join(GOLDEN, f"cfg{i}_full.npz")
    assert os.path.exists(path), f"{path} is missing: python tests/golden/make_goldens.py {i}"
    g = dict(np.load(path))
    w = inputs.config(i)
    P, L, N, iters = w.P, w.L, w.N, w.iters
    assert list(g["meta"]) == [i, P, L, N, iters, w.seed], "the record was written for another workload"
    tag = f"[cfg{i} full run]"
    say(f"\n{tag} P={P} L={L} N={N} iterations={iters}: building the ring")
    x0 = np.broadcast_to(w.x0()[None, :], (P, N))
    ring = evg.Ring.from_workload(w, x0, mailbox_fill=float("nan"))
    del x0
    dg = GpuDigest(ring, w.layer_numel)
    digest_at = {int(k): d for d, k in enumerate(g["digest_iters"])}
    for k in range(iters):
        ring.step(k)
        d = ring.decisions()
        bad = np.argwhere(d["fired"] != g["fired"][k])
        if bad.size:
            r, l = (int(v) for v in bad[0])
            if d["near_tie"][r, l] and g["near_tie"][k][r, l]:
                pytest.fail(f"{tag} iteration {k}: worker {r}, tensor {l} is a near tie on both sides and the "
                            f"decisions differ; regenerate the record with "
                            f"`python tests/golden/make_goldens.py {i} --override {k},{r},{l},{int(d['fired'][r, l] > 0)}`")
            pytest.fail(f"{tag} iteration {k}: decisions differ at (worker, tensor) {bad[:5].tolist()}: "
                        f"norm {d['norm'][r, l]!r} vs {g['norm'][k][r, l]!r}, threshold {g['delta_before'][k][r, l]!r}")
        assert np.array_equal(d["near_tie"], g["near_tie"][k]), f"{tag} iteration {k}: near-tie flags"
        np.testing.assert_allclose(d["norm"], g["norm"][k], rtol=2e-7, atol=1e-37, err_msg=f"{tag} iteration {k}: norms")
        np.testing.assert_allclose(d["delta_before"], g["delta_before"][k], rtol=4e-7, atol=1e-37,
                                   err_msg=f"{tag} iteration {k}: thresholds")
        if w.topk_ppm:
            ih, mh = ring.message_hashes()
            assert np.array_equal(ih, g["idx_hash"][k]), \
                f"{tag} iteration {k}: Top-K index sets differ at {np.argwhere(ih != g['idx_hash'][k])[:5].tolist()}"
            assert np.array_equal(mh, g["msg_hash"][k]), \
                f"{tag} iteration {k}: Top-K values differ at {np.argwhere(mh != g['msg_hash'][k])[:5].tolist()}"
        st = ring.stats()
        got = [st["events_total"], st["value_words"], st["index_words"], st["near_tie_flags"]]
        assert got == [int(v) for v in g["totals"][k]], f"{tag} iteration {k}: running totals {got}"
        if k in digest_at:
            compare_digest(dg, g, digest_at[k], k, say, tag, final=(k == iters - 1))
    st = ring.stats(arrays=True)
    assert np.array_equal(st["events_full_rl"], g["events_full"]) and np.array_equal(st["events_topk_rl"], g["events_topk"])
    assert np.array_equal(st["last_event_iter"], g["last_event_iter"])
    assert np.array_equal(st["valid_l"], g["valid_l"]) and np.array_equal(st["valid_r"], g["valid_r"])
    np.testing.assert_allclose(st["delta"], g["delta"], rtol=4e-7, atol=1e-37)
    assert st["iters"] == iters and st["regular_events"] == P * L * iters
    say(f"{tag} Top-K work granules selected from the arenas instead of their staging slots: {st['chunks_not_staged']} "
        f"of {int(st['events_topk_rl'].astype(np.int64).sum())} Top-K events' granules; library-owned memory "
        f"{st['library_bytes'] / 1e9:.2f} GB")
    say(f"{tag} {st['events_total']} events of {st['regular_events']} "
        f"({100.0 * st['events_total'] / st['regular_events']:.1f} % of the regular algorithm's messages), "
        f"{int(g['totals'][-1][3])} near ties: decisions, messages and parameters equal the oracle's")
