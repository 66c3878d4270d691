"""bench.py on the GPU machine: the JSON line keeps its contract (metric, value, roofline objects measured live,
per-batch figures, the planner's table from dp_profile_layer), and the single-GPU multiplexing run reports
its ladder.  Short runs on a reduced layer list / few steps; no figure is asserted, only presence and sanity."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*flags):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *flags], capture_output=True, text=True, timeout=280)
    assert r.returncode == 0, r.stderr[-2000:]
    return json.loads(r.stdout.strip().splitlines()[-1])


def test_bench_line_contract():
    d = _run("--steps", "2", "--warmup", "1", "--no-cpu-baseline", "--no-glue", "--batches", "2,32", "--layers", "conv1_2,conv3_2,conv4_2,fc7")
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config"):
        assert key in d, key
    assert d["unit"] == "TFLOP/s" and d["n_gpus"] == 1 and d["dtype"] == "bf16" and d["vs_baseline"] is None and "workload" in d["config"]
    assert d["value"] > 0 and abs(d["value"] - d["config"]["flops_per_step"] / d["ms_per_step"] / 1e9) <= 1e-6 * d["value"]
    for n in ("2", "32"):
        pb = d["per_batch"][n]
        assert pb["us"] > 0 and 0 < pb["frac_mfma_peak"] < 1 and pb["us_sum_of_main_kernels"] <= pb["us_sum_of_calls"] * 1.001
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["peak"] == 2500.0 and r["unit"] == "TFLOP/s" and 0 < r["frac"] < 1
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9 and abs(r["achieved"] - r["flops_per_launch_avg"] / r["avg_launch_us"] / 1e6) <= 1e-6 * r["achieved"]
    h = d["roofline_hbm"]
    assert h["bound"] == "hbm" and h["peak"] == 8000.0 and h["unit"] == "GB/s" and 0 < h["frac"] < 1
    assert d["roofline_batch2"]["samples_per_launch"] == 2
    # the planner's table: dp_profile_layer rows per layer and batch
    assert set(d["layer_table_us"]) == {"conv1_2", "conv3_2", "conv4_2", "fc7"} and "dp_profile_layer" in d["layer_table_source"]
    for rows in d["layer_table_us"].values():
        assert set(rows) == {"2", "32"} and all(v > 0 for row in rows.values() for v in row)


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_multiplex_run_reports_its_ladder():
    d = _run("--multiplex", "--steps", "3")
    assert d["unit"] == "TFLOP/s" and d["value"] > 0 and "default priority" in d["config"]["workload"]
    configs = [r["config"] for r in d["ladder"]]
    assert configs[0].startswith("foreground alone") and "background alone" in configs and sum("collocated" in c for c in configs) >= 3
    alone = d["ladder"][0]["fg_step_us"]
    for r in d["ladder"]:
        if "collocated" in r["config"]:
            assert r["fg_step_us"] > 0 and r["bg_tflops"] > 0 and abs(r["fg_slowdown"] - r["fg_step_us"] / alone) < 1e-9
    assert set(d["fg_layer_latency_us"]) >= {"conv1_1", "conv3_2", "fc6", "fc8"}
    assert all(a > 0 and b > 0 for a, b in d["fg_layer_latency_us"].values())
