"""bench.py refuses a run on more than one GPU (no GPU needed to say so)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], cwd=ROOT, capture_output=True,
                         text=True, timeout=300)
    assert out.returncode != 0
    assert "one gpu" in (out.stdout + out.stderr).lower()


def test_traffic_of_the_dominant_kernel_comes_from_the_committed_profile():
    """roofline.traffic is read from profiles/ (rocprofv3 --pmc summary), not typed in: the file must name the
    headline's dominant kernel under the library's launch name and give more bytes than the kernel's own
    algorithmic ones (12 B per entry of the COO part + X and Y once)."""
    sys.path.insert(0, ROOT)
    import bench
    t = bench.traffic_from_profile("spmm_coo")
    assert t is not None and t > 2.3e9
    assert bench.traffic_from_profile("no_such_kernel") is None
