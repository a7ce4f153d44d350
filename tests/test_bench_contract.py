"""bench.py's command line and the JSON line it prints."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""


def load_bench():
    import importlib.util
    spec = importlib.util.spec_from_file_location("evg_bench", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    return bench


def test_counter_figures_come_from_tracked_profiles():
    """bench.py holds no measured constant: roofline.traffic and the VALU instruction count are read
    from profiles/counters_<workload>.json, which records the run they were measured on."""
    from paper_2103_07454_amd import inputs
    bench = load_bench()
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert "MEASURED_TRAFFIC_BYTES" not in src and "MEASURED_VALU" not in src
    for i in (3, 4, 5):
        w = inputs.config(i)
        rec = bench.measured_counters(w.name)
        assert rec is not None, f"profiles/counters_{w.name}.json is missing"
        assert rec["workload"] == w.name and rec["steps"] > 0 and 0.0 <= rec["fraction_fired_topk"] <= 1.0
        upd = rec["kernels"]["k_update"]
        elems = w.P * w.N
        assert 20 * elems < upd["traffic_bytes"] < 60 * elems           # a streaming pass over five arrays
        assert abs(upd["traffic_bytes"] - upd["fetch_bytes"] - upd["write_bytes"]) < 1.0
        assert 0.9 < rec["calibration"]["write_factor"] < 1.1
    assert bench.measured_counters(inputs.config(4).name)["kernels"]["k_update"]["valu_instructions_per_element"] > 50
    assert bench.measured_counters("no_such_workload") is None


@pytest.mark.gpu
def test_json_line_of_a_short_run(monkeypatch, capsys):
    bench = load_bench()
    monkeypatch.setattr(sys, "argv", ["bench.py", "--config", "2", "--steps", "5", "--warmup", "1",
                                      "--no-cpu-baseline"])
    bench.main()                                   # in this process: no second program on the GPU
    lines = [l for l in capsys.readouterr().out.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 1 and d["unit"] == "elements/s"
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "f32"
    assert d["config"]["workload"].startswith("cfg2") and "model" not in d["config"]
    assert abs(d["value"] - d["config"]["P"] * d["config"]["elements_per_worker"] * 5 / (d["ms_per_step"] * 5e-3)) \
        <= 1e-6 * d["value"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12 and r["launches"] == 5
    assert abs(r["achieved"] - r["algorithmic_bytes_per_launch"] / (r["avg_launch_ms"] * 1e-3) / 1e9) <= 1e-6 * r["achieved"]
    # whole-tensor sends: nothing is patched, the line-granular floor is the algorithmic figure
    assert r["line_granular_floor_bytes_per_launch"] >= r["algorithmic_bytes_per_launch"]
    assert r["traffic"] is None and r["traffic_measured_at"] is None      # no counter run is recorded for configuration 2
