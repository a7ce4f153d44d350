"""Planted mistakes: every single-line mutation of the oracle listed here must make at least
one pin test fail.  Each mutant is a copy of oracle/evg_oracle.cpp with one edit, compiled on
the CPU and handed to a child pytest run of the oracle's pin tests through EVG_ORACLE_LIB.
A mutant that survives means a part of the oracle is pinned only against itself."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "evg_oracle.cpp")
PINS = ["tests/test_oracle_generator.py", "tests/test_oracle_method.py", "tests/test_oracle_pins_precision.py"]

# (name, text to find -- must occur exactly once --, replacement)
MUTANTS = [
    # trigger and threshold
    ("ge_to_gt", "(d >= dl)", "(d > dl)"),
    ("slope_off_by_one", "(float)((int64_t)k - (int64_t)o.last_event[s])", "(float)((int64_t)k - (int64_t)o.last_event[s] + 1)"),
    ("horizon_dropped", "o.delta[s] = c.horizon * slope;", "o.delta[s] = slope;"),
    ("forced_first_event_dropped", "bool fire = (c.force_first && k == 0) || (d >= dl);", "bool fire = (d >= dl);"),
    ("history_mean_is_sum", "o.delta[s] = c.horizon * (sum / (float)hst.size());", "o.delta[s] = c.horizon * sum;"),
    ("history_keeps_one_too_many", "if (hst.size() > c.hist_len) hst.erase(hst.begin());", "if (hst.size() > c.hist_len + 1) hst.erase(hst.begin());"),
    # norm
    ("norm_without_sqrt", "d = (float)std::sqrt(acc);", "d = (float)acc;"),
    ("norm_accumulated_in_float", "double acc = 0.0;\n        for (uint64_t j = 0; j < n; ++j) {\n          const float e = xs[j] - hs[j];\n          acc += (double)e * (double)e;",
     "float acc = 0.0f;\n        for (uint64_t j = 0; j < n; ++j) {\n          const float e = xs[j] - hs[j];\n          acc += e * e;"),
    ("norm_difference_accumulated_in_float", "double ax = 0.0, ah = 0.0;", "float ax = 0.0f, ah = 0.0f;"),
    ("norm_difference_without_abs", "d = std::fabs((float)std::sqrt(ax) - (float)std::sqrt(ah));", "d = (float)std::sqrt(ax) - (float)std::sqrt(ah);"),
    # near-tie band
    ("band_ten_times_wider", "< 1e-6f * dl;", "< 1e-5f * dl;"),
    ("band_ten_times_narrower", "< 1e-6f * dl;", "< 1e-7f * dl;"),
    ("band_edge_included", "std::fabs(d - dl) < 1e-6f * dl;", "std::fabs(d - dl) <= 1e-6f * dl;"),
    ("near_ties_not_counted", "if (near) o.near_ties++;", ""),
    ("band_never_flags", "const bool near = std::fabs(d - dl) < 1e-6f * dl;\n      o.near_tie[s] = near;\n      if (near) o.near_ties++;\n      bool fire",
     "bool near = false;\n      bool fire"),
    # sends and ring addressing
    ("neighbours_swapped", "float* toR = &o.mbox_r[left * N + o.off[l]];    // I am", "float* toR = &o.mbox_r[right * N + o.off[l]];    // I am"),
    ("xhat_not_updated_on_whole_send", "          hs[j] = xs[j];\n          if (now) { toR[j] = xs[j]; toL[j] = xs[j]; }\n        }\n        o.fired[s] = 1;",
     "          if (now) { toR[j] = xs[j]; toL[j] = xs[j]; }\n        }\n        o.fired[s] = 1;"),
    ("first_message_not_sent_whole", "if (c.topk_ppm == 0 || first) {", "if (c.topk_ppm == 0) {"),
    ("valid_flag_ignored", "(vl ? (o.mbox_l[base + j] - xv) : 0.0f)", "(o.mbox_l[base + j] - xv)"),
    # Top-K
    ("ties_to_higher_index", ": a < b;", ": a > b;"),
    ("key_is_sum", "c.topk_key == 0 ? xs[j] - hs[j] : xs[j]", "c.topk_key == 0 ? xs[j] + hs[j] : xs[j]"),
    ("k_rounded_down", "(n * (uint64_t)cfg.topk_ppm + 999999ull) / 1000000ull", "(n * (uint64_t)cfg.topk_ppm) / 1000000ull"),
    ("index_fingerprint_unmixed", "o.idx_hash[s] += splitmix64((uint64_t)j);", "o.idx_hash[s] += (uint64_t)j;"),
    ("message_fingerprint_without_values", "splitmix64(((uint64_t)f2u(xs[j]) << 32) | (uint64_t)j)", "splitmix64((uint64_t)j)"),
    ("splitmix_constant", "0xBF58476D1CE4E5B9ull", "0xBF58476D1CE4E5B1ull"),
    # update
    ("mixing_weight", "(float)(1.0 / 3.0)", "0.3f"),
    ("step_sign", "std::fmaf(-c.lr, vn, cns)", "std::fmaf(c.lr, vn, cns)"),
    ("momentum_dropped", "std::fmaf(c.momentum, o.vel[base + j], gp[j])", "gp[j]"),
    # generator
    ("philox_constant", "0xCD9E8D57u", "0xCD9E8D55u"),
    ("sin_cos_swapped", "z[2 * h] = rad * c;", "z[2 * h] = rad * s;"),
    ("decay_off_by_one", "std::pow(cfg.decay, (double)k)", "std::pow(cfg.decay, (double)k + 1)"),
    ("spike_counter_moved", "{0u, 0xFFFFFFFFu, (uint32_t)k, r}", "{0u, 0xFFFFFFFEu, (uint32_t)k, r}"),
    ("spike_draw_from_other_word", "return uniform01(w[0]) < cfg.spike_prob;", "return uniform01(w[1]) < cfg.spike_prob;"),
    ("student_t_degrees", "std::sqrt(3.0f * (exp_poly(y) - 1.0f))", "std::sqrt(2.0f * (exp_poly(y) - 1.0f))"),
    ("student_t_exponent", "0.666666687f * -log_poly(u)", "0.5f * -log_poly(u)"),
    ("student_t_angle_reuses_the_radius_word", "v = uniform01(w[2 * i + 1]);", "v = uniform01(w[2 * i]);"),
    ("student_t_blocks_overlap", "(uint32_t)(2 * (j0 >> 2) + b)", "(uint32_t)((j0 >> 2) + b)"),
    ("student_t_radius_without_minus_one", "(exp_poly(y) - 1.0f)", "exp_poly(y)"),
    ("exp_series_term", "p = std::fmaf(r, p, 0.166666672f);", "p = std::fmaf(r, p, 0.125f);"),
    # delayed delivery and the other reading of a Top-K event
    ("delayed_messages_land_at_once", "const bool now = c.delivery_delay == 0;", "const bool now = true;"),
    ("xhat_reset_ignored", "if (c.xhat_reset)\n", "if (false)\n"),
    # final average
    ("average_divides_by_one_less", "(float)(acc / (double)o.cfg.P)", "(float)(acc / (double)(o.cfg.P - 1))"),
]


def build_and_run(job):
    name, old, new, workdir = job
    text = open(SRC).read()
    if text.count(old) != 1:
        return name, "edit", f"pattern occurs {text.count(old)} times"
    src = os.path.join(workdir, f"{name}.cpp")
    lib = os.path.join(workdir, f"lib_{name}.so")
    with open(src, "w") as f:
        f.write(text.replace(old, new))
    cc = subprocess.run(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-w", "-o", lib, src],
                        capture_output=True, text=True)
    if cc.returncode != 0:
        return name, "compile", cc.stderr[-400:]
    env = dict(os.environ, EVG_ORACLE_LIB=lib)
    run = subprocess.run([sys.executable, "-m", "pytest", *PINS, "-x", "-q", "-p", "no:cacheprovider"],
                         cwd=ROOT, env=env, capture_output=True, text=True)
    last = (run.stdout.strip().splitlines() or [""])[-1]
    return name, "killed" if run.returncode == 1 else "survived" if run.returncode == 0 else "error", last


@pytest.mark.timeout(900)
def test_every_planted_mistake_fails_a_pin(tmp_path):
    jobs = [(n, o, r, str(tmp_path)) for (n, o, r) in MUTANTS]
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(build_and_run, jobs))
    report = "\n".join(f"{n}: {s} ({d})" for n, s, d in results)
    print(report)
    bad = [(n, s, d) for n, s, d in results if s != "killed"]
    assert not bad, f"planted mistakes that no pin notices (or that did not apply):\n{bad}\n\nall:\n{report}"
