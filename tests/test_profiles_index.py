"""profiles/INDEX.md is what bench.py reads its counter figures from (`roofline.traffic`,
`mfma_busy_pct`): every row must say what the rocprofv3 summary it names says, and
bench.py's look-up must find the rows of the configurations it reports."""
import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")


def _rows():
    rows = bench.profile_index()
    assert rows, "profiles/INDEX.md has no rows"
    return rows


def test_every_index_row_matches_the_summary_it_names():
    for r in _rows():
        path = os.path.join(PROFILES, r["file"])
        assert os.path.exists(path), r["file"]
        text = open(path).read()
        # the commands that made the summary run committed files only
        assert "rocprofv3 --kernel-trace --stats" in text and "bench.py --config" in text and "_work" not in text
        avg = float(re.search(r"calls \d+\s+average ([\d.]+) us", text).group(1))
        assert abs(avg - float(r["avg launch us"])) < 0.006, r["file"]
        traffic = int(re.search(r"traffic_bytes_per_launch = (\d+)", text).group(1))
        assert traffic == int(r["traffic bytes per launch"]), r["file"]
        ratio = float(re.search(r"read traffic / algorithmic bytes = ([\d.]+)", text).group(1))
        assert abs(ratio - float(r["read / algorithmic"])) < 0.0006, r["file"]
        busy = float(re.search(r"MFMA utilisation = busy / \(1024 SIMDs x kernel cycles\): ([\d.]+) %", text).group(1))
        assert abs(busy - float(r["MFMA busy %"])) < 0.06, r["file"]
        pct = float(re.search(r"GB/s = ([\d.]+) % of the 8 TB/s HBM peak", text).group(1))
        assert abs(pct - float(r["% of 8 TB/s"])) < 0.06, r["file"]
        assert f"Kernel  : ssrnn::{r['kernel']}<" in text, r["file"]
        assert f"Weights : {r['weights']}" in text, r["file"]
        assert ("--flags 1" in text) == (r["schedule"] == "per-stage"), r["file"]
        assert ("--packed" in text) == (r["weights"] == "packed"), r["file"]
        assert f"--T {r['T']} " in text and f"--config {r['workload'][:2]} " in text, r["file"]


def test_bench_finds_the_rows_it_reports():
    rows = _rows()
    # headline point in both schedules, the other profiled block sizes of the headline workload, configuration 5
    for key in (("C4", 4, "row-major", "wavefront"), ("C4", 4, "row-major", "per-stage"), ("C4", 1, "row-major", "wavefront"),
                ("C4", 1, "row-major", "per-stage"), ("C5", 16, "packed", "wavefront"), ("C5", 64, "packed", "wavefront"),
                ("C5", 256, "packed", "wavefront")):
        r = bench.profile_row(*key, rows)
        assert r is not None, key
        assert int(r["traffic bytes per launch"]) > 0
    assert bench.profile_row("C4", 3, "row-major", "wavefront", rows) is None


def test_read_traffic_stays_close_to_the_algorithmic_bytes():
    """Traffic well above the algorithmic bytes means wasted re-reads."""
    for r in _rows():
        assert 0.98 <= float(r["read / algorithmic"]) <= 1.10, (r["file"], r["read / algorithmic"])
