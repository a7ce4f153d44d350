"""Writes tests/golden/cfgN_full.npz: the CPU oracle's record of a benchmark configuration
run at FULL size for its FULL iteration count.

Only `oracle/` (the CPU oracle) and `paper_2103_07454_amd.inputs` (seeded inputs, no method
arithmetic) are imported: nothing here touches the HIP library, so every stored value is the
oracle's.  The GPU test tests/test_gpu_golden_full.py steps the HIP path through the same run
and compares against this record.

    python tests/golden/make_goldens.py 3 4 5            (about 15 / 25 / 35 minutes, one thread each;
                                                          configuration 5 needs about 22 GB of RAM)
    python tests/golden/make_goldens.py 5 --override 17,3,12,1
        re-runs with the decision of (iteration 17, worker 3, tensor 12) forced to "fire" where
        the oracle itself flags a near tie (|norm - delta| < 1e-6 delta): the parity rule allows
        the two sides to differ there, and the record must then follow the HIP path's decision.

What is stored (S = P*L tests per iteration):
  fired[k, r, l]        0 silent, 1 whole tensor sent, 2 Top-K message sent
  near_tie[k, r, l]     the 1e-6 band flag
  norm, delta_before    the norm each test used and the threshold it was compared with
  idx_hash, msg_hash    per Top-K message: sum over its entries of splitmix64(index) and of
                        splitmix64(value bits << 32 | index), modulo 2^64 (0 where none)
  totals[k]             running events_total, value_words, index_words, near_tie_flags
  digest_iters          iterations after which the five arrays were fingerprinted
  dg_<array>_bits[d, r, l]    sum_j bits(v_j) * w_j mod 2^64,  w_j = ((j+1) * 0x9E3779B97F4A7C15) | 1
  dg_<array>_sum, _maxabs     float64 sum and float32 max |v| per (worker, tensor)
  dg_<array>_sample[d, :]     the array's values at `sample_index` (positions in the unpadded
                              [P, N] layout); `final_<array>_sample` / `final_sample_index` hold a
                              larger sample after the last iteration
  delta, last_event_iter, events_full, events_topk, valid_l, valid_r   tables after the last iteration
"""
from __future__ import annotations

import argparse
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2103_07454_amd import inputs  # noqa: E402

ARRAYS = ("x", "xhat", "vel", "mbox_l", "mbox_r")
DIGEST_EVERY = 10
SAMPLE = 8192            # values kept per array at every digest
FINAL_SAMPLE = 131072    # values kept per array after the last iteration
WEIGHT_MUL = np.uint64(0x9E3779B97F4A7C15)


def position_weights(n: int) -> np.ndarray:
    j = np.arange(1, n + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return (j * WEIGHT_MUL) | np.uint64(1)


def fingerprint(arr: np.ndarray, numel: np.ndarray, weights):
    """arr: [P, N] float32.  Returns (bits [P, L] uint64, sum [P, L] float64, maxabs [P, L] float32)."""
    P = arr.shape[0]
    L = numel.size
    bits = np.zeros((P, L), np.uint64)
    sums = np.zeros((P, L), np.float64)
    maxabs = np.zeros((P, L), np.float32)
    off = np.concatenate([[0], np.cumsum(numel.astype(np.int64))])
    u = arr.view(np.uint32)
    with np.errstate(over="ignore"):
        for l in range(L):
            sl = slice(int(off[l]), int(off[l + 1]))
            w = weights[l]
            for r in range(P):
                bits[r, l] = (u[r, sl].astype(np.uint64) * w).sum(dtype=np.uint64)
            sums[:, l] = arr[:, sl].sum(axis=1, dtype=np.float64)
            maxabs[:, l] = np.abs(arr[:, sl]).max(axis=1)
    return bits, sums, maxabs


def run(i: int, overrides, out_dir: str, iters_cap=None):
    w = inputs.config(i)
    iters = w.iters if iters_cap is None else min(w.iters, iters_cap)
    P, L, N = w.P, w.L, w.N
    numel = w.layer_numel
    t0 = time.time()
    print(f"[cfg{i}] {w.name}: P={P} L={L} N={N} iterations={iters}", flush=True)
    x0 = inputs.replicate(w.x0(), P)
    orc = oracle.Oracle.from_workload(w, x0)
    del x0
    weights = [position_weights(int(n)) for n in numel]
    rng = np.random.Generator(np.random.Philox(key=1000 + i))
    sample_index = np.sort(rng.integers(0, P * N, size=SAMPLE, dtype=np.int64))
    final_index = np.sort(rng.integers(0, P * N, size=FINAL_SAMPLE, dtype=np.int64))
    ov = {}
    for (k, r, l, dec) in overrides:
        ov.setdefault(k, []).append((r, l, dec))

    rec = {n: [] for n in ("fired", "near_tie", "norm", "delta_before", "idx_hash", "msg_hash", "totals")}
    dg = {f"dg_{a}_{q}": [] for a in ARRAYS for q in ("bits", "sum", "maxabs", "sample")}
    digest_iters = []
    for k in range(iters):
        override = None
        if k in ov:
            override = np.full(P * L, -1, np.int8)
            for (r, l, dec) in ov[k]:
                override[r * L + l] = dec
        orc.step(k, override=override)
        d = orc.decisions()
        ih, mh = orc.message_hashes()
        tot = orc.totals()
        for name in ("fired", "near_tie", "norm", "delta_before"):
            rec[name].append(d[name].copy())
        rec["idx_hash"].append(ih)
        rec["msg_hash"].append(mh)
        rec["totals"].append(np.array([tot["events_total"], tot["value_words"], tot["index_words"],
                                       tot["near_tie_flags"]], np.uint64))
        if override is not None:
            for (r, l, dec) in ov[k]:
                if not d["near_tie"][r, l]:
                    raise SystemExit(f"override ({k},{r},{l}) is not a near tie for the oracle: refused")
        last = k == iters - 1
        if (k + 1) % DIGEST_EVERY == 0 or last:
            digest_iters.append(k)
            for a in ARRAYS:
                arr = orc.state(a)
                b, s, m = fingerprint(arr, numel, weights)
                dg[f"dg_{a}_bits"].append(b)
                dg[f"dg_{a}_sum"].append(s)
                dg[f"dg_{a}_maxabs"].append(m)
                dg[f"dg_{a}_sample"].append(arr.reshape(-1)[sample_index].copy())
                if last:
                    dg[f"final_{a}_sample"] = arr.reshape(-1)[final_index].copy()
                del arr
        print(f"[cfg{i}] iteration {k + 1}/{iters}  fired {float((d['fired'] > 0).mean()):.3f}  "
              f"near ties so far {tot['near_tie_flags']}  {time.time() - t0:.0f} s", flush=True)

    tb = orc.tables()
    out = {k: np.stack(v) for k, v in rec.items()}
    for k, v in dg.items():
        out[k] = np.stack(v) if isinstance(v, list) else v
    out["digest_iters"] = np.array(digest_iters, np.int64)
    out["sample_index"] = sample_index
    out["final_sample_index"] = final_index
    out["overrides"] = np.array(overrides, np.int64).reshape(-1, 4)
    for name in ("delta", "last_event_iter", "events_full", "events_topk", "valid_l", "valid_r"):
        out[name] = tb[name]
    out["meta"] = np.array([i, P, L, N, iters, w.seed], np.int64)
    suffix = "" if iters == w.iters else f"_first{iters}"
    path = os.path.join(out_dir, f"cfg{i}_full{suffix}.npz")
    np.savez_compressed(path, **out)
    print(f"[cfg{i}] wrote {path} ({os.path.getsize(path) / 1e6:.1f} MB) in {time.time() - t0:.0f} s", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("configs", type=int, nargs="+", choices=[1, 2, 3, 4, 5])
    ap.add_argument("--override", action="append", default=[],
                    help="k,r,l,decision (0/1): follow this decision where the oracle flags a near tie")
    ap.add_argument("--iters", type=int, default=None, help="stop early (file name says so)")
    ap.add_argument("--out", default=HERE)
    a = ap.parse_args()
    overrides = [tuple(int(v) for v in o.split(",")) for o in a.override]
    oracle.build()
    for i in a.configs:
        run(i, overrides, a.out, a.iters)


if __name__ == "__main__":
    main()
