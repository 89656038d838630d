"""bench.py's contract: one JSON line with the agreed keys; more than one GPU is refused."""
from __future__ import annotations

import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and not r.stdout.strip()


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_contract_keys():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "96", "--warmup", "8", "--layers", "4"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 96 and d["warmup"] == 8 and d["unit"] == "stream-tokens/s"
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and "workload" in d["config"] and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9 and 0 < rf["frac"] < 1
    assert rf["kernel_samples"] >= 8 and rf["kernel_samples_in_timed_region"] >= 2 and rf["kernel_us_min"] <= rf["kernel_us_median"]
    # the read-only form of the same launch is the measured ceiling: faster than the real launch
    assert rf["measured_read_us"] is not None and rf["measured_read_us"] < rf["kernel_us"]
    assert abs(rf["frac_of_measured_read"] - rf["measured_read_us"] / rf["kernel_us"]) < 1e-6
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["unit"] == d["unit"] and cb["sample"]
    assert d["value"] > 100 * cb["value"]
    assert d["parity_vs_oracle"]["rel_l2"] <= 1e-2 and d["parity_vs_oracle"]["max_abs"] <= 2e-2
