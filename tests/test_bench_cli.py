"""Host-only checks of bench.py's command line."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout == ""


def test_source_digest_is_stable_and_names_the_kernel_sources():
    sys.path.insert(0, ROOT)
    import bench
    d = bench.csrc_digest()
    assert len(d) == 16 and d == bench.csrc_digest()
    assert set(bench.MEASURED_TRAFFIC["MB_per_step"]) <= set(bench.PHASE_KERNELS)
    assert set(bench.PHASE_LAUNCHES) == set(bench.PHASE_KERNELS)
