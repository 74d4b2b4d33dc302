"""Host-side checks of bench.py that need no GPU: it refuses more than one GPU with a message, and
its HBM-traffic and matrix-core figures are read from the committed rocprofv3 summary."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "single-GPU" in p.stderr and p.stdout.strip() == ""


def test_counter_figures_come_from_the_committed_profile():
    """bench.py's HBM-traffic and matrix-core counter figures are read from the rocprofv3 summary under
    profiles/ (they need separate --pmc runs), not typed into the script: the reader finds every
    (mode, GEMM) pair, and the machine-readable lines agree with the summary's own table."""
    sys.path.insert(0, ROOT)
    import bench
    assert not hasattr(bench, "MEASURED_TRAFFIC")
    prof = bench.load_counter_profile()
    text = open(os.path.join(ROOT, bench.COUNTER_PROFILE)).read()
    for mode in ("streaming", "resident", "resident_separate_passes", "large_m"):
        for k in ("gemm1", "gemm2"):
            e = prof[(mode, k)]
            assert set(e) == {"fetch_bytes", "write_bytes", "mfma_busy_frac", "mfma_issued_over_algorithmic"}
            m = re.search(r"^\s+%s\s+%s: HBM bytes per launch\s+([\d.]+) MB .*?busy ([\d.]+) %% .*?algorithmic = ([\d.]+)$" % (mode, k), text, re.M)
            assert m, (mode, k)
            assert abs((e["fetch_bytes"] + e["write_bytes"]) / 1e6 - float(m.group(1))) <= 0.06
            assert abs(100 * e["mfma_busy_frac"] - float(m.group(2))) <= 0.06
            assert abs(e["mfma_issued_over_algorithmic"] - float(m.group(3))) <= 0.006
            assert 0 < e["mfma_busy_frac"] < 1 and e["mfma_issued_over_algorithmic"] >= 1.0
    assert bench.load_counter_profile(os.path.join(ROOT, "profiles", "no-such-file.txt")) == {}
