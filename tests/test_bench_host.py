"""Host-side checks of bench.py that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_comes_from_the_committed_counter_summary():
    sys.path.insert(0, ROOT)
    import bench
    t = bench.traffic_from_profile("7b_block")
    # the gemm_y slot moves at least its algorithmic bytes (x 64 MB + W_eff 32 MB in, y 64 MB out for the smallest
    # projection) and the summary's own rows add up to the figure
    assert t is not None and 1.5e8 < t < 5e9
    rows = [l for l in open(bench.TRAFFIC_PROFILE) if l.startswith("|") and "nt_gemm_kernel" in l.split("|")[1] and
            ("<256, 256, 0, false, false, 2, true>" in l or "<256, 128, 0, false, false, 2, true>" in l)]
    assert len(rows) == 2
    assert bench.traffic_from_profile("1b_block") is None  # not profiled: null, never a stale literal


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2 and "ONE GPU" in res.stderr
