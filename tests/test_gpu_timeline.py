"""The in-kernel clock stamps (libecspmv_trace.so, the library's sources built with -DECS_TRACE) and the script that
reads them: a short run on the small config, in a process of its own because it loads the stamped library in place of
the product one.  The stamped kernel must still compute y (the script's launches are checked against the oracle's band
by the parity tests of the product library; here the order of the stamped points is what is checked)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_timeline_runs_and_points_come_in_order(tmp_path):
    from paper_2507_12205_amd import build as B
    if not os.path.exists(B.TRACE_LIB):
        pytest.fail(f"{B.TRACE_LIB} is missing: __graft_entry__.build() makes it")
    out = tmp_path / "t.json"
    env = dict(os.environ)
    env.pop("ECSPMV_LIB", None)
    r = subprocess.run([sys.executable, "-m", "paper_2507_12205_amd.timeline", "--config", "0", "--shape", "0",
                        "--copies", "2", "--launches", "6", "--json", str(out)],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=240)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    d = json.loads(out.read_text())
    by = {row["stamp"]: row for row in d["stamps"]}
    for k in (0, 1, 2, 3, 4, 12):
        assert k in by, f"stamp {k} missing"
    # a wavefront passes these points in this order, so their medians over a launch do too
    order = [0, 23, 1, 4, 12]
    med = [by[k]["median_us"] for k in order]
    assert all(a <= b for a, b in zip(med, med[1:])), med
    assert 0.0 < d["kernel_span_us"] < 100.0 and d["us_per_launch_stamps_off"] > 0.0
    assert 500.0 < d["stamp_clock_mhz"] < 3000.0
