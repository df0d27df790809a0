"""CPU-side checks of bench.py's contract that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr
    assert res.stdout.strip() == ""


def test_bench_reads_the_committed_traffic_figures():
    sys.path.insert(0, ROOT)
    import bench
    fwd = bench._traffic_from_profiles("carousel_forward_config4_n4096_B4096_f32")
    bwd = bench._traffic_from_profiles("carousel_backward_config4_n4096_B4096_f32")
    assert fwd is not None and 1e9 < fwd < 3e9
    assert bwd is not None and 1e10 < bwd < 5e10
    assert bench._traffic_from_profiles("no_such_kernel") is None
