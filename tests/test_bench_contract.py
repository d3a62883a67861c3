"""bench.py's contract with its caller: the refusal of more than one GPU (CPU), and on a GPU the one JSON
line with the fields a driver reads, internally consistent."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args, timeout=600):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=timeout, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert r.returncode != 0 and r.stdout.strip() == ""
    assert "ONE GPU" in r.stderr


@pytest.mark.gpu
def test_default_line_carries_the_contract_fields():
    r = run_bench("--gpus", "1", "--steps", "8", "--warmup", "2")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, "exactly one JSON line on stdout"
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 8 and d["warmup"] == 2 and d["higher_is_better"] is True
    assert d["unit"] == "tokens/s" and d["dtype"] == "bf16" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert "workload" in d["config"] and "model" not in d["config"]
    # value is rows per step over the step time
    assert abs(d["value"] - d["config"]["rows"] / (d["ms_per_step"] * 1e-3)) <= 1e-6 * d["value"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9 and 0.3 < rf["frac"] < 1.0
    assert abs(rf["achieved"] - rf["algorithmic_bytes"] / (rf["kernel_ms"] * 1e-3) / 1e9) <= 1e-6 * rf["achieved"]
    assert rf["kernel_ms"] < d["ms_per_step"]            # the kernel is part of the step
    assert rf["traffic"] is None or 0.9 < rf["traffic"] / rf["algorithmic_bytes"] < 1.5
    pp = d["roofline_pp"]
    assert pp["bound"] == "mfma" and pp["unit"] == "TFLOP/s" and pp["peak"] == 2500.0 and 0.05 < pp["frac"] < 1.0
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "tokens/s" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
    assert d["value"] > 100 * cb["value"]
