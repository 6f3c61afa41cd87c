"""Host-side checks of the measurement scripts' contract (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT,
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = _run("--gpus", "2")
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_without_a_gpu_the_bench_fails_loudly_instead_of_falling_back():
    import torch
    if torch.cuda.is_available():
        return                                   # on a GPU machine the real run is the round-end bench
    p = _run("--steps", "1", "--warmup", "0")
    assert p.returncode != 0 and "no GPU" in p.stderr and p.stdout.strip() == ""


def test_traffic_figure_comes_from_the_committed_profile():
    sys.path.insert(0, ROOT)
    import bench
    t = bench._read_traffic("k_gather_k_direct_relu_ffn.txt")
    assert t is not None and 1.5e8 < t < 4e8     # FETCH + WRITE bytes per launch of the headline kernel
    assert bench._read_traffic("no_such_profile.txt") is None
