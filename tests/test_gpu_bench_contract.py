"""bench.py's one-line contract, on the smallest configuration (needs a GPU)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, cwd=ROOT,
                          timeout=280)


def test_bench_prints_one_json_line_with_the_agreed_fields():
    r = _run("--config", "1", "--steps", "3", "--warmup", "1", "--cpu-seconds", "1", "--cpu-workers", "2", "--no-other-configs")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["metric"] == "decode layer-steps/sec" and d["unit"] == "layer-steps/s" and d["higher_is_better"] is True
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["scaling"] == "weak" and d["data"] == "synthetic"
    assert d["vs_baseline"] is None and d["dtype"] in ("f16", "bf16")
    assert d["value"] > 0 and abs(d["value"] * d["ms_per_step"] - 1e3) < 1e-6 * 1e3
    assert "workload" in d["config"] and "model" not in d["config"] and d["config"]["workload"].startswith("cfg1")
    roof = d["roofline"]
    assert roof["bound"] == "hbm" and roof["unit"] == "GB/s" and roof["peak"] == 8000.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12 and 0 < roof["frac"] < 1 and "traffic" in roof
    assert roof["launch_us_median_min_max"][1] <= roof["launch_us_median_min_max"][0] <= roof["launch_us_median_min_max"][2]
    assert abs(roof["avg_launch_ms"] * 1e3 - roof["launch_us_median_min_max"][0]) < 1e-9
    res = d["gpu_resident"]
    for leg in ("replay_one_query", "rotating"):
        assert res[leg]["misses"] == 0 and res[leg]["repeats"] >= 3 and res[leg]["launches_per_repeat"] >= 20
        assert res[leg]["us_min"] <= res[leg]["us_per_launch_median"] <= res[leg]["us_max"]
    assert abs(roof["achieved"] - res["rotating"]["GBps"]) < 1e-9
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["unit"] == "layer-steps/s" and cpu["value"] > 0 and cpu["cores"] == 2 and cpu["sample"]
    assert "configs" not in d


def test_bench_reports_the_other_configurations_too():
    """The default run adds one entry per other configuration of the benchmark definition."""
    r = _run("--config", "1", "--steps", "3", "--warmup", "1", "--cpu-seconds", "0")
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads([l for l in r.stdout.splitlines() if l.strip()][-1])
    assert sorted(d["configs"]) == ["cfg2", "cfg3", "cfg4", "cfg5"]
    for name, c in d["configs"].items():
        assert c["workload"].startswith(name) and c["layer_steps_per_s"] > 0 and 0 <= c["hit_rate"] <= 1
        g = c["gpu_resident"]
        assert g["misses"] == 0 and 0 < g["frac_of_hbm_peak"] < 1 and g["us_min"] <= g["us_per_launch_median"] <= g["us_max"]
        assert c["step_form"].startswith("one launch")
    assert "gpu_resident_layers_overlapped" in d["configs"]["cfg2"] and "gpu_resident_layers_overlapped" in d["configs"]["cfg4"]
    for name in ("cfg2", "cfg4"):                          # the decode step of a many-layer configuration, end to end
        e = d["configs"][name]["decode_step_of_8_layers"]
        assert e["layers"] == 8 and e["max_abs_output_difference"] == 0.0
        assert 0 < e["overlapped"]["ms_per_layer_step"] <= 1.05 * e["one_by_one"]["ms_per_layer_step"]
    assert "cpu_baseline" not in d


def test_bench_reshapes_a_configuration_on_request():
    """--page-size keeps the budget's and the cache's tokens; the stored counter readings of the
    configuration as defined are not reported for the reshaped one."""
    r = _run("--config", "1", "--page-size", "8", "--steps", "3", "--warmup", "1", "--cpu-seconds", "0", "--no-other-configs")
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads([l for l in r.stdout.splitlines() if l.strip()][-1])
    assert " page=8 " in d["config"]["workload"] and "k=128 pages (1024 tokens)" in d["config"]["workload"]
    assert "cache=512 pages/unit (100%" in d["config"]["workload"]
    assert d["roofline"]["traffic"] is None and d["roofline"]["traffic_note"]
    assert d["gpu_resident"]["rotating"]["misses"] == 0 and d["value"] > 0


def test_bench_refuses_more_than_one_gpu():
    r = _run("--gpus", "2")
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
