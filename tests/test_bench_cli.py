"""bench.py's command line where no GPU is needed: more than one GPU is refused with a message, and without a GPU
the benchmark stops instead of falling back to anything that runs on the host."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, env=None):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300, env=env)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_without_a_gpu_the_benchmark_stops():
    env = dict(os.environ, HIP_VISIBLE_DEVICES="", CUDA_VISIBLE_DEVICES="", ROCR_VISIBLE_DEVICES="")
    r = _run("--steps", "1", "--warmup", "0", env=env)
    assert r.returncode != 0
    assert "no GPU" in r.stderr and r.stdout.strip() == ""
