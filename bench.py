#!/usr/bin/env python3
"""Benchmark of the EventGraD per-iteration parameter path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5]

One "step" is one evg_step: trigger tests, sends (whole tensors or Top-K
messages) and the fused averaging + SGD update for all P simulated workers.
The default workload is configuration 5 (P = 64 ring workers, ResNet-18-shaped
parameter list, adaptive thresholds, Top-K 10 %, 100 iterations).  W warm-up
steps run first; the state is then re-initialised (untimed) and K steps,
iterations 0..K-1 of the configuration, are timed with inputs resident in HBM.
The roofline, phase and per-step figures come from a second, instrumented run of
the same K iterations.

Prints one JSON line: throughput in parameter-elements/s, the roofline figures
of the dominant kernel (the fused update pass, timed with HIP events on the
stream it runs on), per-step percentiles, what a plain triad reaches on the same
box, and the CPU oracle's throughput on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published peak, GB/s
# Algorithmic bytes of the update pass per element: reads x, mbox_l, mbox_r, vel,
# xhat and writes x, vel (fp32) = 28; with Top-K it also reads the three messages
# (8 rho per fired element) and scatters them into xhat and both mailboxes (12 rho).
UPDATE_BYTES_PER_ELEM = 28
UPDATE_TOPK_BYTES_PER_FIRED_ELEM_PER_RHO = 20

# Counter figures (HBM bytes of one k_update launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE;
# vector-ALU instructions per element from SQ_INSTS_VALU) are not typed in here: they are read from
# profiles/counters_<workload>.json, which `python -m paper_2103_07454_amd.rocprof_summary` writes from
# the profiler's output together with the step count and fired share they were measured at.
# What the chip can issue: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second.
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12


def measured_counters(workload):
    """The tracked counter summary of this workload, or None if none has been recorded."""
    path = os.path.join(ROOT, "profiles", f"counters_{workload}.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    rec["file"] = os.path.relpath(path, ROOT)
    return rec


def cpu_baseline(inputs, w, seconds_hint=20.0):
    """The oracle as it stands, single thread, on a bounded sample of the same
    workload: a ring of 4 of its workers (the oracle's cost per element does not depend on the
    ring size), first iterations -- as many as fit 10-30 s, so that the two all-fire iterations
    0 and 1 weigh as little as the bound allows."""
    import oracle
    P = min(4, w.P)
    ws = w.scaled(P=P)
    iters = min(20, max(2, int(4.5e8 // (P * ws.N))))     # about 10-30 s of single-thread work
    x0 = inputs.replicate(ws.x0(), P)
    orc = oracle.Oracle.from_workload(ws, x0)
    t0 = time.perf_counter()
    for k in range(iters):
        orc.step(k)
    dt = time.perf_counter() - t0
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), model)
    except OSError:
        pass
    return {"value": P * ws.N * iters / dt, "unit": "elements/s", "cores": 1, "kind": "oracle",
            "sample": f"{w.name} with P={P} ring workers, iterations 0..{iters - 1}, {dt:.1f} s",
            "host_cpu": model, "host_logical_cpus": os.cpu_count()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--seed", type=int, default=None,
                    help="seed of initial parameters and gradient streams (default: the configurations' own)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-phase-timers", action="store_true")
    ap.add_argument("--trigger-kind", type=int, default=0,
                    help="0 = norm of the drift (default, the benchmark configurations); "
                         "1 = difference of the norms")
    ap.add_argument("--delivery-delay", type=int, default=0,
                    help="1 = messages land after the iteration's updates (not a benchmark configuration)")
    ap.add_argument("--plain-sgd", action="store_true",
                    help="momentum 0, the paper's optimiser (not a benchmark configuration): the velocity "
                         "arena is then neither read nor written")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of captured evg_step_next calls instead of K evg_step calls "
                         "(same iterations; for the launch-bound small rings)")
    ap.add_argument("--graph-steps", type=int, default=1,
                    help="iterations recorded into the one graph (must divide --steps)")
    ap.add_argument("--xhat-reset", type=int, default=0,
                    help="1 = a Top-K event resets the whole tensor's xhat (not a benchmark configuration)")
    ap.add_argument("--topk-ppm", type=int, default=None,
                    help="another Top-K share, in parts per million (not a benchmark configuration: shows how "
                         "the update pass's distance to its algorithmic bytes depends on the share sent)")
    ap.add_argument("--diag-grad-buffer", action="store_true",
                    help="diagnostic only (not the named workload): gradients from a fixed device buffer")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the parameter path of all P simulated workers on ONE GPU; "
              "--gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2103_07454_amd import evg, inputs

    w = inputs.config(args.config) if args.seed is None else inputs.config(args.config, args.seed)
    if args.plain_sgd:
        w = w.scaled(momentum=0.0)
    if args.topk_ppm is not None:
        w = w.scaled(topk_ppm=args.topk_ppm)
    x0 = w.x0()[None, :]                       # common start; uploaded once per worker slice
    x0 = np.broadcast_to(x0, (w.P, w.N))

    gbuf = None

    side = torch.cuda.Stream() if args.graph else None

    def make():
        if side is not None:
            with torch.cuda.stream(side):
                return evg.Ring.from_workload(w, x0, chunk_elems=args.chunk, trigger_kind=args.trigger_kind,
                                              delivery_delay=args.delivery_delay, xhat_reset=args.xhat_reset,
                                              stream=side)
        if args.diag_grad_buffer:
            return evg.Ring.from_workload(w, x0, chunk_elems=args.chunk, grad_mode=evg.GRAD_BUFFER,
                                          trigger_kind=args.trigger_kind, delivery_delay=args.delivery_delay,
                                          xhat_reset=args.xhat_reset)
        return evg.Ring.from_workload(w, x0, chunk_elems=args.chunk, trigger_kind=args.trigger_kind,
                                      delivery_delay=args.delivery_delay, xhat_reset=args.xhat_reset)

    ring = make()
    if args.diag_grad_buffer:
        gbuf = torch.randn_like(ring.x) * 1e-4
    for k in range(args.warmup):
        ring.step(k, gbuf)
    ring.synchronize()
    ring.close()
    del ring
    torch.cuda.empty_cache()

    # timed region: fresh state, iterations 0..K-1, no instrumentation of any kind
    ring = make()
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        assert args.steps % args.graph_steps == 0
        with torch.cuda.graph(graph, stream=side):
            for _ in range(args.graph_steps):
                ring.step_next()               # recorded, not run: the replays are iterations 0..K-1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps // args.graph_steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        assert ring.stats()["iters"] == args.steps
    else:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            ring.step(k, gbuf)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0

    # the same K iterations once more from a fresh state, now with the library's phase
    # timers and one event per step (these cost a few microseconds per step, which is
    # why they stay out of the region that `value` is computed from)
    per_step = not args.no_phase_timers
    marks = []
    if per_step:
        ring.close()
        del ring
        torch.cuda.empty_cache()
        ring = make()
        ring.timing(True)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        torch.cuda.synchronize()
        for k in range(args.steps):
            marks[k].record(ring.stream)
            ring.step(k, gbuf)
        marks[args.steps].record(ring.stream)
        torch.cuda.synchronize()

    st = ring.stats(arrays=True)
    phases = ring.timing_read() if not args.no_phase_timers else {}
    elems = w.P * w.N
    numel = w.layer_numel.astype(np.float64)
    rho = w.topk_ppm / 1e6
    f_full = float((st["events_full_rl"].astype(np.float64) * numel[None, :]).sum() / (elems * args.steps))
    f_topk = float((st["events_topk_rl"].astype(np.float64) * numel[None, :]).sum() / (elems * args.steps))
    step_bytes_per_elem = (28 if w.momentum != 0.0 else 20) + 16 * f_full + 8 * f_topk + 28 * rho * f_topk
    out = {
        "metric": "param_elements_per_s_fused_trigger_consensus_update",
        "value": elems * args.steps / dt,
        "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name + ("+DIAG_GRAD_BUFFER" if args.diag_grad_buffer else "")
                   + ("+NORM_DIFF_TRIGGER" if args.trigger_kind else "")
                   + ("+DELAYED_DELIVERY" if args.delivery_delay else "")
                   + ("+XHAT_RESET" if args.xhat_reset else "") + ("+PLAIN_SGD" if args.plain_sgd else "")
                   + (f"+TOPK_PPM_{args.topk_ppm}" if args.topk_ppm is not None else ""), "P": w.P, "tensors": w.L, "elements_per_worker": w.N, "seed": w.seed,
                   "threshold": "adaptive" if w.thr_mode else "fixed", "topk_ppm": w.topk_ppm,
                   "chunk_elems": args.chunk or (2048 if 5 * 4 * w.P * evg.padded_numel(w.layer_numel) <= (128 << 20)
                                                 else 8192),
                   "launch": f"replays of one captured HIP graph of {args.graph_steps} iteration(s)" if args.graph else "one evg_step call per iteration",
                   "fraction_fired_full": f_full, "fraction_fired_topk": f_topk,
                   "messages_pct_of_regular": 100.0 * st["events_total"] / max(1, st["regular_events"]),
                   "communication_pct_of_regular":
                       100.0 * (st["value_words"] + st["index_words"]) / max(1, st["regular_words"])},
        "library_owned_bytes": st["library_bytes"],
        "topk_chunks_not_staged": st["chunks_not_staged"],
        "step_algorithmic_bytes_per_element": step_bytes_per_elem,
        "step_achieved_GBps": step_bytes_per_elem * elems * args.steps / dt / 1e9,
        "step_frac_of_hbm_peak": step_bytes_per_elem * elems * args.steps / dt / 1e9 / HBM_PEAK_GBS,
    }
    if phases:
        ms_upd, n_upd = phases["update"]
        avg_ms = ms_upd / max(1, n_upd)
        per_elem = UPDATE_BYTES_PER_ELEM + UPDATE_TOPK_BYTES_PER_FIRED_ELEM_PER_RHO * rho * f_topk
        if w.momentum == 0.0:
            per_elem -= 8          # plain SGD: no velocity read or write
        if args.trigger_kind == 1 and not w.topk_ppm:
            per_elem -= 4          # xhat is not read: its norm is a scalar per tensor
        upd_bytes = per_elem * elems
        achieved = upd_bytes / (avg_ms * 1e-3) / 1e9
        # What the dense-mailbox semantics cost at the granularity memory is written in: the dense
        # 28 (or fewer) bytes per element (a tensor that was sent whole has its xhat written instead
        # of read: the same 4 bytes), each message read by its sender and both receivers (3 x 8 bytes
        # per entry), and the write-back of every aligned 64-byte group of xhat and of the two
        # mailboxes that holds a sent entry.  With K of n entries sent, spread evenly, a 16-float
        # group holds one with probability 1 - (1 - K/n)^16.
        dense = per_elem - UPDATE_TOPK_BYTES_PER_FIRED_ELEM_PER_RHO * rho * f_topk
        ev_topk = st["events_topk_rl"].astype(np.float64).sum(axis=0)        # per tensor, all workers and steps
        K = np.array([max(1, min(int(n), -(-int(n) * w.topk_ppm // 1_000_000))) if w.topk_ppm else 0
                      for n in w.layer_numel], np.float64)
        share = K / numel
        dirty = 1.0 - (1.0 - share) ** 16
        floor = dense * elems + float((ev_topk * numel * (12 * dirty + 24 * share)).sum()) / args.steps
        counters = measured_counters(w.name) if not (args.diag_grad_buffer or args.trigger_kind or args.delivery_delay
                                                     or args.xhat_reset or args.plain_sgd or args.seed is not None
                                                     or args.topk_ppm is not None) else None
        upd_counters = (counters or {}).get("kernels", {}).get("k_update", {})
        traffic = upd_counters.get("traffic_bytes")
        out["roofline"] = {"kernel": "k_update", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                           "traffic": traffic,
                           "traffic_measured_at": None if traffic is None else {
                               "file": counters["file"], "steps": counters["steps"],
                               "fraction_fired_topk": counters["fraction_fired_topk"],
                               "fraction_fired_full": counters["fraction_fired_full"]},
                           "avg_launch_ms": avg_ms, "launches": n_upd,
                           "algorithmic_bytes_per_launch": upd_bytes,
                           "line_granular_floor_bytes_per_launch": floor,
                           "floor_over_algorithmic": floor / upd_bytes,
                           "traffic_over_floor": None if traffic is None else traffic / floor,
                           "achieved_on_floor_GBps": floor / (avg_ms * 1e-3) / 1e9}
        valu = upd_counters.get("valu_instructions_per_element")
        if valu is not None and w.dist == 1:
            # Student-t gradients: the generator, not memory, bounds the pass
            ops = valu * elems / (avg_ms * 1e-3) / 1e12
            out["roofline"] = {"kernel": "k_update", "bound": "alu", "achieved": ops, "peak": ALU_PEAK_TLANEOPS,
                               "unit": "T lane-instructions/s", "frac": ops / ALU_PEAK_TLANEOPS, "traffic": traffic,
                               "avg_launch_ms": avg_ms, "launches": n_upd,
                               "algorithmic_bytes_per_launch": upd_bytes,
                               "line_granular_floor_bytes_per_launch": floor,
                               "valu_instructions_per_element": valu,
                               "valu_measured_at": {"file": counters["file"]},
                               "hbm_achieved_GBps": achieved, "hbm_frac": achieved / HBM_PEAK_GBS}
        out["phase_ms_per_step"] = {p: ms / max(1, args.steps) for p, (ms, n) in phases.items()}
        # the other HBM-bound phases against the same peak, on their share of the lower-bound bytes:
        # whole sends move 12 B per fired element here (xhat := x rides in the update pass), the
        # Top-K selection one key pass over x and xhat (8 B), packing writes the 8 rho message
        alg = {"send_full": 12 * f_full, "topk_select": 8 * f_topk, "topk_send": 8 * rho * f_topk}
        out["phase_frac_of_hbm_peak"] = {
            p: b * elems / (phases[p][0] / max(1, args.steps) * 1e-3) / 1e9 / HBM_PEAK_GBS
            for p, b in alg.items() if phases[p][0] > 0 and b > 0}
    if per_step:
        # iterations 0 and 1 fire every tensor (forced first event, then a zero threshold)
        ms = np.array([marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps)])
        out["step_ms"] = {"median": float(np.median(ms)), "p10": float(np.percentile(ms, 10)),
                          "p90": float(np.percentile(ms, 90)), "first_two": [float(v) for v in ms[:2]]}
    # the final model average (last line of Algorithm B): one pass over x of all workers
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ring.average()
    ev0.record(ring.stream)
    avg_reps = 5
    for _ in range(avg_reps):
        evg._check(evg.lib().evg_average(ring._h, ring.xhat.data_ptr()))   # xhat is scratch now
    ev1.record(ring.stream)
    torch.cuda.synchronize()
    avg_ms = ev0.elapsed_time(ev1) / avg_reps
    out["final_average"] = {"ms": avg_ms, "achieved_GBps": 4.0 * elems / (avg_ms * 1e-3) / 1e9}
    ring.close()
    del ring
    torch.cuda.empty_cache()
    # what a plain streaming kernel reaches on this machine: c = a + s*b over arrays of one arena's size
    n_tri = max(elems, 1 << 26)
    ta, tb, tc = (torch.full((n_tri,), float(i), device="cuda") for i in range(3))
    torch.add(ta, tb, alpha=0.5, out=tc)
    ev0.record()
    for _ in range(avg_reps):
        torch.add(ta, tb, alpha=0.5, out=tc)
    ev1.record()
    torch.cuda.synchronize()
    tri = 12.0 * n_tri / (ev0.elapsed_time(ev1) / avg_reps * 1e-3) / 1e9
    out["stream_triad"] = {"kind": "torch c = a + 0.5 b, fp32", "elements": n_tri, "GBps": tri,
                           "frac_of_hbm_peak": tri / HBM_PEAK_GBS}
    if "roofline" in out and out["roofline"]["bound"] == "hbm":
        out["roofline"]["frac_of_triad"] = out["roofline"]["achieved"] / tri
    del ta, tb, tc
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inputs, w)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
