"""Host-side pieces of bench.py that need no GPU: the measured-traffic figure comes from the committed
counter summary of the workload, with the commit it was collected at, and is absent (not invented) for a
workload that has no summary; more than one GPU is refused with a message."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_traffic_figure_is_read_from_the_committed_summary():
    val, source = bench.measured_traffic("llada_64k", 0.10)
    text = open(os.path.join(ROOT, "profiles", "pmc_traffic_llada_64k_keep10.md")).read()
    assert val == float(re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text).group(1))
    sha = re.search(r"collected_at_commit:\s*(\w+)", text).group(1)
    assert sha in source and "pmc_traffic_llada_64k_keep10.md" in source
    # between the algorithmic bytes of a launch (Q, O, the selected K and V rows once, the column numbers) and
    # what re-fetching every selected row for every query block would cost
    algorithmic = 32 * (2 * 65536 * 128 + 2 * 6553 * 128) * 2 + 32 * 4 * 6553
    assert algorithmic < val < 30 * algorithmic


def test_no_summary_means_no_figure():
    val, source = bench.measured_traffic("llada_4k", 0.10)
    assert val is None and "no committed counter summary" in source


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
