"""CPU-only checks of bench.py's command line: more than one GPU is refused with a message, and the
traffic figure is only reported for the GEMM source it was measured on."""
import hashlib
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert p.returncode == 2
    assert "one GPU" in p.stderr
    assert p.stdout.strip() == ""


def test_traffic_figure_is_tied_to_the_gemm_source():
    sys.path.insert(0, ROOT)
    import bench
    src = os.path.join(ROOT, "paper_2407_19775_amd", "csrc", "gemm_kernels.hip")
    same = hashlib.sha256(open(src, "rb").read()).hexdigest() == bench.GEMM_TRAFFIC_SOURCE_SHA256
    assert (bench.gemm_traffic() is not None) == same
    if same:
        assert bench.gemm_traffic() == bench.GEMM_TRAFFIC_BYTES_PER_LAUNCH
