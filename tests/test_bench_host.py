"""Host-side checks of bench.py that need no GPU: it refuses more than one GPU with a message, and
its stored HBM-traffic figures are the ones of the committed rocprofv3 summary."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "single-GPU" in p.stderr and p.stdout.strip() == ""


def test_traffic_table_matches_the_committed_profile():
    sys.path.insert(0, ROOT)
    import bench
    text = open(os.path.join(ROOT, "profiles", "grouped_ffn_switch-base-128.hbm_traffic.txt")).read()
    measured = {}
    for mode, kern, shape, mb in re.findall(r"^\s+(resident|streaming)\s+(gemm[12]) \(grouped_gemm_nt<([^>]*)>\)\s*:\s*([\d.]+) MB measured", text, re.M):
        measured[(mode, kern, shape)] = float(mb) * 1e6
    wl = "switch-base-128-T16384"

    def one(mode, kern, fused):
        """The figure of the only tile shape that (mode, kernel) ran with."""
        hits = [v for (m, k, shape), v in measured.items() if m == mode and k == kern and ("fused" in shape) == fused]
        assert len(hits) == 1, (mode, kern, fused, hits)
        return hits[0]

    for mode, kern in (("resident", "gemm1"), ("resident", "gemm2"), ("resident_fused", "gemm1"), ("resident_fused", "gemm2"),
                       ("streaming", "gemm1")):
        got = bench.MEASURED_TRAFFIC[(wl, mode, kern)]
        want = one(mode.replace("_fused", ""), kern, mode.endswith("_fused"))
        assert abs(got - want) <= 1e-3 * want, (mode, kern, got, want)
    # the streaming GEMM 2 figure is the launch-weighted mean of its two tile shapes
    narrow, wide = measured[("streaming", "gemm2", "128x128")], measured[("streaming", "gemm2", "128x256")]
    got = bench.MEASURED_TRAFFIC[(wl, "streaming", "gemm2")]
    assert min(narrow, wide) < got < max(narrow, wide)
    n_narrow, n_wide = (int(re.search(r"streaming\s+gemm2 \(grouped_gemm_nt<%s>\).*?(\d+) dispatches" % shape, text).group(1))
                        for shape in ("128x128", "128x256"))
    assert abs(got - (n_narrow * narrow + n_wide * wide) / (n_narrow + n_wide)) <= 2e-3 * got
