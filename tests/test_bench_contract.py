"""Host-side checks of bench.py's command line: more than one GPU is refused with a message, and the options parse."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_help_lists_the_contract_flags():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 0
    for flag in ("--gpus", "--steps", "--warmup", "--launch", "--delta-bits", "--config"):
        assert flag in r.stdout


import json

import pytest


@pytest.mark.gpu
def test_bench_line_on_the_small_config():
    """One JSON line with the contract's keys, the roofline and CPU-baseline objects, the launch floor, and every
    timed leg checked against the oracle (config 0, a few steps: the numbers mean nothing at this size)."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "0", "--steps", "5", "--warmup", "2",
                        "--no-other-configs"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-3000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["unit"] == "GB/s" and d["value"] > 0
    assert "workload" in d["config"] and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3 and "traffic" in rf
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1 and cb["sample"]
    assert d["parity_checked"]["all_ok"] is True and len(d["parity_checked"]["legs"]) >= 3
    assert d["paper_context"]["speedup_over_best_fp16_baseline"]["max"] == 6.44 and "RTX" in d["paper_context"]["hardware"]
    fl = d["launch_floor"]
    assert 0.5 < fl["empty_launch_256x1024_us"] < 50.0 and fl["step_of_lone_launches_us"] > 0
