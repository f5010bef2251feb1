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


def test_measured_traffic_table_matches_the_committed_counter_summary():
    """bench.py's table of measured HBM bytes per launch is typed in from the counter runs summarised under
    profiles/: the two must not drift apart."""
    import re
    sys.path.insert(0, ROOT)
    import bench
    rows = {}
    for line in open(os.path.join(ROOT, "profiles", "hbm_traffic_cfg3_llavanext_b8.txt")):
        m = re.match(r"^(\w+)\s+(\d+)\s+([\d.]+)\s+([\d.]+)\s+([\d.]+)\s", line)
        if m:
            rows[m.group(1)] = (float(m.group(3)), float(m.group(4)), float(m.group(5)))
    assert rows, "no counter rows found in the summary"
    for name, nbytes in bench.MEASURED_HBM_TRAFFIC_BYTES.items():
        assert name in rows, f"{name} is in bench.py's table but not in the summary"
        fetch_kib, write_kib, mb = rows[name]
        assert abs((2.0 * fetch_kib + write_kib) * 1024 - nbytes) <= 0.001 * nbytes + 2048, name
        assert abs(mb - nbytes / 1e6) <= 0.06, name
