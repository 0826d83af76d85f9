"""The default bench run measures the attention kernel's HBM bytes per launch itself (two child runs under
rocprofv3 --pmc).  Collected late: it is the slowest bench test and leans on a tool outside the repository."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_default_workload_reports_live_traffic():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "3", "--warmup", "1", "--no-cpu-baseline", "--no-also"],
                         capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert res.returncode == 0, res.stderr[-2000:]
    r = json.loads([l for l in res.stdout.splitlines() if l.startswith("{")][0])
    rf = r["roofline"]
    assert rf["traffic"] is not None
    if "no live measurement" in rf["traffic_source"]:
        pytest.skip(rf["traffic_source"])
    assert "rocprofv3 --pmc" in rf["traffic_source"] and "child runs" in rf["traffic_source"]
    # K/V pages, page table, Q, new K/V and output are the algorithmic bytes; split-KV partials and the plan come on top
    assert 1.0 <= rf["traffic"] / rf["algorithmic_bytes_per_launch"] <= 1.08, rf
