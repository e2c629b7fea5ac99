"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "one GPU" in (res.stdout + res.stderr)


def test_profiled_figures_are_read_from_the_committed_summaries():
    sys.path.insert(0, ROOT)
    import bench
    t = bench.read_profile_value(os.path.join(ROOT, "profiles", "fused_chain_hbm_traffic_70b_r8_decode.md"), "traffic_bytes_per_launch")
    assert t is not None and 15e9 < t < 21e9, t   # bytes per launch = per decode step (chained); algorithmic: 17.4e9
    assert bench.read_profile_value(os.path.join(ROOT, "profiles", "no_such_file.md"), "traffic_bytes_per_launch") is None
    us = bench.read_profile_value(os.path.join(ROOT, "profiles", "fused_chain_kernel_70b_r8_decode.md"), "rocprofv3_avg_launch_us")
    assert us is not None and 2000 < us < 5000, us   # one launch per step
