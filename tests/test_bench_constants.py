"""bench.py quotes two kinds of figures it cannot measure in-process: HBM-side traffic per launch (rocprofv3 byte
counters) and hardware peaks.  The traffic figures must be the ones the committed profile summary states, for the
commit it names; this test reads the summary's table independently and compares."""
import os
import re
import subprocess

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _table_value(text, label):
    for line in text.splitlines():
        if line.startswith("| " + label):
            cells = [c.strip() for c in line.strip("|").split("|")]
            return float(cells[2]), float(cells[3])
    raise AssertionError(f"row {label!r} not found")


def test_traffic_constants_are_those_of_the_profile_summary():
    text = open(bench.PROFILE_TRAFFIC).read()
    want = {("C5/p05/s60", "gather"): _table_value(text, "prefill attention, gather mode"),
            ("C5/p05/s60", "rebase"): _table_value(text, "prefill attention, telescoped mode"),
            ("C4/p05/s57", "decode"): _table_value(text, "decode step kernel")}
    assert set(bench.MEASURED_TRAFFIC_BYTES) == set(want)
    for key, (fetch_mib, write_mib) in want.items():
        assert bench.MEASURED_TRAFFIC_BYTES[key] == (fetch_mib + write_mib) * 2 ** 20
        assert fetch_mib > 0 and write_mib > 0
    # the summary names the commit its counters were taken at, and bench.py passes that on
    m = re.search(r"^Counters taken at commit `([0-9a-f]{7,40})`", text, flags=re.M)
    assert m and bench.TRAFFIC_FROM_COMMIT == m.group(1)
    known = subprocess.run(["git", "cat-file", "-t", m.group(1)], cwd=ROOT, capture_output=True, text=True)
    if known.returncode == 0:                                   # (a checkout without history cannot tell)
        assert known.stdout.strip() == "commit"


def test_published_peaks():
    assert bench.PEAK_HBM_GBS == 8000.0 and bench.PEAK_MFMA_BF16_TFLOPS == 2500.0
    assert bench.PEAK_VALU_F32_TFLOPS == 157.3 and abs(bench.FMA_MIX_ISSUE_TFLOPS - 157.3 / 2) < 0.06
