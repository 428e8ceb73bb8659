"""bench.py's command-line contract, without a GPU: it refuses more than one GPU with a message, and the
recorded HBM traffic of the dominant kernel is read from the committed counter summary."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_recorded_traffic_comes_from_the_committed_profile():
    sys.path.insert(0, ROOT)
    import bench
    v = bench.recorded_traffic("gemm_bf16_pipe_k_verify")
    assert v is not None and 1e8 < v < 1e10
    assert bench.recorded_traffic("no_such_kernel") is None
