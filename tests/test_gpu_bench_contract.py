"""bench.py end to end on the smallest workload: one JSON line with the fields the measurement contract
names, the dominant kernel timed inside the timed region, the oracle timed beside it.  Run as a child process, as the driver runs it."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True,
                          text=True, timeout=280)


@pytest.mark.timeout(300)
@pytest.mark.parametrize("extra", [(), ("--graph",), ("--variant", "pa", "--overselect", "4")],
                         ids=["eager", "graph-replay", "alg1-with-second-round"])
def test_bench_prints_one_json_line_with_the_contract_fields(extra):
    p = run_bench("--workload", "C1", "--steps", "4", "--warmup", "2", "--cpu-sample-d", "200000",
                  "--no-vram-precondition", *extra)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["unit"] == "coords/s" and j["n_gpus"] == 1 and j["steps"] == 4 and j["warmup"] == 2
    assert j["dtype"] == "f32" and j["data"] == "synthetic" and j["vs_baseline"] is None and j["higher_is_better"] is True
    assert "workload" in j["config"] and "model" not in j["config"]
    assert abs(j["value"] - j["config"]["d"] / (j["ms_per_step"] * 1e-3)) <= 1e-6 * j["value"]
    r = j["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s" and r["avg_launch_ms"] > 0.0
    assert r["launches_per_step"] >= 1.0 and r["kernel"] in j["kernels_ms_per_step"]
    if r["achieved"] is not None:
        assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12
    assert r["peak_measured_copy"] > 100.0 and "traffic_from" in r
    assert min(j["ms_per_step_min_max"]) <= j["ms_per_step_median"] <= max(j["ms_per_step_min_max"])
    c = j["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] == 1 and c["value"] > 0.0 and c["unit"] == "coords/s" and c["sample"]
    ct = j["cpu_baseline_threads"]
    assert ct["kind"] == "oracle" and ct["cores"] >= 1 and ct["value"] > 0.0 and ct["same_result_as_single_thread"] is True


@pytest.mark.timeout(300)
def test_bench_times_both_memory_states_in_one_run():
    p = run_bench("--workload", "C1", "--steps", "3", "--warmup", "1", "--no-cpu-baseline")
    assert p.returncode == 0, p.stderr[-2000:]
    j = json.loads([ln for ln in p.stdout.splitlines() if ln.strip()][-1])
    assert j["config"]["vram_preconditioned"] is True
    f = j["fresh_memory_state"]
    assert f["ms_per_step"] > 0.0 and f["value"] > 0.0

