"""The instrumented build (libpsk_trace.so): bench.py --cu-trace runs in a process of its own (a process loads one
of the two libraries), on a small matrix; every workgroup must have left a record and the busy times must be sane."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_cu_trace_report_on_a_small_matrix():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "expskew", "--skew-rows", "4096",
                        "--skew-nnz", "400000", "--cu-trace"], capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    rec = json.loads([l for l in r.stdout.splitlines() if l.startswith("{")][-1])
    names = [s["schedule"] for s in rec["schedules"]]
    assert any("position cut" in n for n in names) and any("wave per row" in n for n in names)
    for s in rec["schedules"]:
        assert s["workgroups"] > 0 and 1 <= s["compute_units"] <= 256
        assert s["max_over_mean"] >= 1.0 and s["cu_busy_us"]["max"] <= s["span_us"] + 0.02
    cut = next(s for s in rec["schedules"] if "position cut" in s["schedule"])
    assert cut["workgroups"] == -(-400000 // 2048) or abs(cut["workgroups"] - 400000 // 2048) <= 2


def test_plain_build_has_no_trace():
    import paper_2001_00532_amd as psk

    assert psk.lib().psk_cu_trace_set(None, 0) == 5          # PSK_ERR_UNSUPPORTED in libpsk.so
