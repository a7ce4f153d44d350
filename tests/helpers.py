"""Lock-step comparison of the HIP path with the CPU oracle (used by the GPU tests)."""
import numpy as np

ARENAS = ("x", "xhat", "vel", "mbox_l", "mbox_r")
REL_TOL = 1e-5   # max-abs-normalised bound on fp32 parameters after a full run


def rel_err(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    scale = np.abs(b).max()
    return float(np.abs(a - b).max() / scale) if scale > 0 else float(np.abs(a - b).max())


def masked_mailboxes(ring_or_oracle, valid, numel):
    """Mailbox arenas with never-written tensors blanked (their contents are undefined)."""
    out = {}
    off = np.concatenate([[0], np.cumsum(np.asarray(numel, np.int64))])
    for name, key in (("mbox_l", "valid_l"), ("mbox_r", "valid_r")):
        a = ring_or_oracle.state(name).copy()
        v = valid[key]
        for r, l in zip(*np.nonzero(v == 0)):
            a[r, off[l]:off[l + 1]] = 0
        out[name] = a
    return out


def lockstep(ring, orc, iters, *, grads=None, gpu_grads=None, sample_messages=32, seed=0,
             check_every=None, progress=None, say=print, norm_rtol=2e-7, norm_abs_of_x=None):
    """Steps both sides through ``iters`` iterations.  After every iteration the
    decisions must agree exactly; a disagreement is tolerated only where both
    sides flag a near tie (|norm - delta| < 1e-6 delta), in which case the oracle
    follows the GPU's decision.  Returns a report dict.

    norm_rtol: relative bound on the tested norms and thresholds (drift-norm trigger: both sides
    sum exact double products and differ by summation order only).  norm_abs_of_x: for the
    norm-difference trigger, whose tested quantity | ||x|| - ||xhat|| | is a difference of two
    rounded norms and so carries an absolute error of a few float spacings of ||x||: the bound is
    norm_abs_of_x * ||x|| per (worker, tensor)."""
    rng = np.random.default_rng(seed)
    replayed = 0
    numel = np.asarray(orc._numel, np.int64)
    xnorm_max = None
    for k in range(iters):
        if norm_abs_of_x is not None:
            xs = orc.state("x").astype(np.float64)
            off = np.concatenate([[0], np.cumsum(numel)])
            xn = np.stack([np.sqrt((xs[:, off[l]:off[l + 1]] ** 2).sum(axis=1)) for l in range(numel.size)], axis=1)
            xnorm_max = xn if xnorm_max is None else np.maximum(xnorm_max, xn)
        ring.step(k, grad=None if gpu_grads is None else gpu_grads(k))
        gd = ring.decisions()
        override = np.where(gd["near_tie"] != 0, (gd["fired"] > 0).astype(np.int8), np.int8(-1)).astype(np.int8)
        orc.step(k, grad=None if grads is None else grads(k), override=override.ravel())
        od = orc.decisions()
        bad = gd["fired"] != od["fired"]
        assert not bad.any(), (f"iteration {k}: unflagged decision mismatch at {np.argwhere(bad)[:5].tolist()} "
                               f"gpu norm {gd['norm'][bad][:5]} oracle norm {od['norm'][bad][:5]} "
                               f"delta {od['delta_before'][bad][:5]}")
        replayed += int(((od["near_tie"] != 0) & (gd["near_tie"] != 0)).sum())
        # the 1e-6 band is the only licence for a disagreement, so both sides must agree on where
        # it lies (a flag may differ only where the norms themselves differ in their last bit)
        nt_diff = (gd["near_tie"] != 0) != (od["near_tie"] != 0)
        assert not (nt_diff & (gd["norm"] == od["norm"]) & (gd["delta_before"] == od["delta_before"])).any(), \
            f"iteration {k}: near-tie flags differ at {np.argwhere(nt_diff)[:5].tolist()}"
        if getattr(ring, "topk_ppm", 0):
            # every Top-K message of the iteration, through its fingerprints
            gih, gmh = ring.message_hashes()
            oih, omh = orc.message_hashes()
            assert np.array_equal(gih, oih), f"iteration {k}: Top-K index sets differ at {np.argwhere(gih != oih)[:5].tolist()}"
            assert np.array_equal(gmh, omh), f"iteration {k}: Top-K message values differ at {np.argwhere(gmh != omh)[:5].tolist()}"
            assert ((gih != 0) == (gd["fired"] == 2)).all()
        # norms agree to summation-order rounding; thresholds likewise
        if norm_rtol is not None:
            np.testing.assert_allclose(gd["norm"], od["norm"], rtol=norm_rtol, atol=1e-37, equal_nan=True)
            np.testing.assert_allclose(gd["delta_before"], od["delta_before"], rtol=2 * norm_rtol, atol=1e-37)
        if norm_abs_of_x is not None:
            err = np.abs(gd["norm"].astype(np.float64) - od["norm"].astype(np.float64))
            assert (err <= norm_abs_of_x * xn + 1e-37).all(), (k, float((err / np.maximum(xn, 1e-300)).max()))
            # a threshold is h times a mean of tested norms, each divided by an iteration count >= 1
            # (Eq. 3; h <= 2 in every test that uses this bound), plus the rounding of that mean
            err = np.abs(gd["delta_before"].astype(np.float64) - od["delta_before"].astype(np.float64))
            bound = 2 * norm_abs_of_x * xnorm_max + 4e-7 * np.abs(od["delta_before"].astype(np.float64)) + 1e-37
            assert (err <= bound).all(), k
        if sample_messages:
            rs, ls = np.nonzero(gd["fired"] == 2)
            if rs.size:
                pick = rng.choice(rs.size, size=min(sample_messages, rs.size), replace=False)
                for q in pick:
                    gi, gv = ring.message(int(rs[q]), int(ls[q]))
                    oi, ov = orc.message(int(rs[q]), int(ls[q]))
                    assert np.array_equal(gi, oi), f"iteration {k}: Top-K indices differ for {(rs[q], ls[q])}"
                    assert np.array_equal(gv, ov)
        if check_every and (k + 1) % check_every == 0:
            for name in ("x", "xhat") + (("vel",) if getattr(ring, "momentum", 1.0) != 0.0 else ()):
                assert rel_err(ring.state(name), orc.state(name)) <= REL_TOL, (k, name)
        if progress and (k + 1) % progress == 0:
            say(f"  lockstep iteration {k + 1}/{iters}")
    rep = {"near_tie_pairs": replayed, "bitwise": {}, "rel": {}}
    tb = orc.tables()
    gs = ring.stats(arrays=True)
    assert np.array_equal(gs["valid_l"], tb["valid_l"]) and np.array_equal(gs["valid_r"], tb["valid_r"])
    assert np.array_equal(gs["events_full_rl"], tb["events_full"])
    assert np.array_equal(gs["events_topk_rl"], tb["events_topk"])
    assert np.array_equal(gs["last_event_iter"], tb["last_event_iter"])
    if norm_rtol is not None:
        np.testing.assert_allclose(gs["delta"], tb["delta"], rtol=2 * norm_rtol, atol=1e-37)
    tot = orc.totals()
    for key in ("events_total", "value_words", "index_words", "bytes_sent", "nonfinite_norms", "iters"):
        assert gs[key] == tot[key], (key, gs[key], tot[key])
    if norm_rtol is not None and replayed == 0:
        assert gs["near_tie_flags"] == tot["near_tie_flags"], (gs["near_tie_flags"], tot["near_tie_flags"])
    gm = masked_mailboxes(ring, gs, numel)
    om = masked_mailboxes(orc, tb, numel)
    for name in ARENAS:
        if name == "vel" and getattr(ring, "momentum", 1.0) == 0.0:
            # plain SGD: the library leaves its velocity arena at zero, the oracle's holds the last
            # gradient.  That gradient is still checked: x' = fma(-lr, g, c) with c equal on both
            # sides, so the bitwise comparison of x below fails if the two sides drew different g
            assert not ring.state("vel").any()
            continue
        g = gm[name] if name in gm else ring.state(name)
        o = om[name] if name in om else orc.state(name)
        rep["bitwise"][name] = bool(np.array_equal(g, o))
        rep["rel"][name] = rel_err(g, o)
        assert rep["rel"][name] <= REL_TOL, (name, rep["rel"][name])
    return rep
