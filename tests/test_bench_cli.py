"""bench.py argument handling that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True)
    assert run.returncode != 0
    assert "ONE GPU" in run.stderr and not run.stdout.strip()


def test_without_a_gpu_the_benchmark_says_so_and_prints_no_line():
    """No CPU fallback: on a machine without a GPU bench.py stops before any
    measurement (on a GPU machine this test has nothing to check)."""
    import torch
    if torch.cuda.is_available():
        return
    for extra in ([], ["--workload", "8x1000", "--single-launch", "1"], ["--variant", "stream"]):
        run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *extra],
                             capture_output=True, text=True)
        assert run.returncode == 3, (extra, run.stderr[-300:])
        assert "no GPU" in run.stderr and not run.stdout.strip()


def test_stored_traffic_figure_is_keyed_by_the_kernel_sources():
    """roofline.traffic is a stored counter reading keyed by a hash of the kernel
    sources (comments dropped): the bench line carries it only for the kernels
    it was taken with, and null once they have changed."""
    sys.path.insert(0, ROOT)
    import bench
    K, D = 32, 25_557_032
    for (name, stamp), value in bench.MEASURED_TRAFFIC.items():
        assert name == "resnet50x32" and len(stamp) == 16
        assert 0.99 < value / (4.0 * D * (5 * (K - 1) + 1)) < 1.05
    assert len(bench.kernel_source_hash()) == 16
    assert bench.MEASURED_TRAFFIC.get(("resnet50x32", "0" * 16)) is None
