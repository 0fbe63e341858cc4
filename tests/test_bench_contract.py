"""bench.py's behaviour that can be checked without a GPU: more than one GPU is refused with a message, and
without a GPU the benchmark refuses to run (the HIP path has no CPU fallback)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300, env={**os.environ, "HIP_VISIBLE_DEVICES": "", "CUDA_VISIBLE_DEVICES": ""})


def test_more_than_one_gpu_is_refused():
    r = run_bench("--gpus", "2")
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_no_gpu_means_no_result():
    r = run_bench("--steps", "1", "--warmup", "0")
    assert r.returncode == 3 and "no GPU" in r.stderr and r.stdout.strip() == ""
