"""bench.py prints one JSON line with the fields its callers rely on."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + list(args), capture_output=True, text=True,
                          timeout=300, cwd=ROOT)
    return proc


def test_one_json_line_with_roofline_and_cpu_baseline():
    proc = run_bench("--steps", "5", "--warmup", "2", "--cpu-seconds", "1", "--also", "c2,c1_bwd", "--also-warmup", "3")
    assert proc.returncode == 0, proc.stderr[-2000:]
    lines = [ln for ln in proc.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["unit"] == "tokens/s"
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["config"]["workload"].startswith("c1") and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12 and 0.0 < r["frac"] < 1.0
    assert abs(d["value"] - 8192 * 1e3 / d["ms_per_step"]) / d["value"] < 1e-6   # tokens per step over time per step
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == "tokens/s" and c["cores"] >= 1 and c["value"] > 0 and c["sample"]
    assert d["parity_rel_err"] <= 2e-2
    assert r["frac_wall_clock"] <= r["frac"] * 1.001 and r["traffic_source"].startswith("stored")
    # every further workload carries the same roofline object, its own step and warm-up counts, and (where the
    # matrix cores are used) the MFMA figure
    assert set(d["also"]) == {"c2", "c1_bwd"}
    for name, e in d["also"].items():
        ro = e["roofline"]
        for key in ("bound", "kernel", "achieved", "peak", "unit", "frac", "traffic", "kernel_ms_avg"):
            assert key in ro, (name, key)
        assert ro["kernel_ms_avg"] > 0 and 0.0 < ro["frac"] < 1.0 and e["warmup"] == 3 and e["steps"] == 10
    assert 0.0 < d["also"]["c2"]["mfma"]["frac"] < 1.0 and "mfma" not in d["also"]["c1_bwd"]


def test_yardstick_workload_prints_a_roofline_line_without_cpu_baseline():
    proc = run_bench("--workload", "strip128", "--steps", "5", "--warmup", "2")
    assert proc.returncode == 0, proc.stderr[-2000:]
    d = json.loads(proc.stdout.strip())
    assert "hyena_stream_gate" in d["roofline"]["kernel"] and 0.0 < d["roofline"]["frac"] < 1.0
    assert "cpu_baseline" not in d and d["config"]["workload"].startswith("strip128")


def test_sharded_workload_times_the_shard_entry_point_and_keeps_parity():
    proc = run_bench("--workload", "c2_shards", "--steps", "5", "--warmup", "2", "--settle", "0", "--cpu-seconds", "1")
    assert proc.returncode == 0, proc.stderr[-2000:]
    d = json.loads(proc.stdout.strip())
    assert "hyena_mr_fwd_shard x 4" in d["roofline"]["kernel"] and 0.0 < d["roofline"]["frac"] < 1.0
    assert d["roofline"]["traffic"] is None and d["parity_rel_err"] <= 2e-2


def test_shape_overrides_change_the_named_workload_and_drop_the_stored_traffic():
    proc = run_bench("--workload", "li2", "--batch", "2", "--width", "2048", "--seq-len", "2048", "--steps", "5",
                     "--warmup", "2", "--settle", "0", "--cpu-seconds", "1")
    assert proc.returncode == 0, proc.stderr[-2000:]
    d = json.loads(proc.stdout.strip())
    assert "B=2 L=2048 D=2048" in d["config"]["workload"] and d["roofline"]["traffic"] is None
    assert "also" not in d and d["parity_rel_err"] <= 2e-2
    assert d["roofline"]["algorithmic_bytes_per_launch"] == 8.0 * 2 * 2048 * 2048


def test_backward_of_the_chain_runs_as_a_workload_with_parity():
    proc = run_bench("--workload", "c4_bwd", "--batch", "1", "--seq-len", "2048", "--steps", "3", "--warmup", "1",
                     "--settle", "0", "--cpu-seconds", "1")
    assert proc.returncode == 0, proc.stderr[-2000:]
    d = json.loads(proc.stdout.strip())
    assert "hyena_chain_bwd" in d["roofline"]["kernel"] and d["parity_rel_err"] <= 2e-2


def test_more_than_one_gpu_is_refused_with_a_message():
    proc = run_bench("--gpus", "2")
    assert proc.returncode != 0
    assert "one" in proc.stderr and "not supported" in proc.stderr
    assert proc.stdout.strip() == ""
