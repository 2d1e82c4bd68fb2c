"""bench.py's command line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    for extra_env, args in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "4"}, [])):
        env = dict(os.environ, **extra_env)
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                           env=env, timeout=120)
        assert r.returncode == 2
        assert "ONE GPU" in r.stderr and not r.stdout.strip()


def test_measured_traffic_is_tied_to_the_kernel_sources():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.measured_traffic("no such workload") is None
    got = bench.measured_traffic("cfg2")
    # either the figure taken with exactly these sources, or nothing at all
    assert got is None or 7.85e9 < got < 7.9e9
