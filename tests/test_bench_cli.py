"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    # one GPU only: no sharding, no collectives; the benchmark says so instead of running
    r = _run("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert r.returncode == 2
    assert "one gpu" in r.stderr.lower() and r.stdout.strip() == ""


def test_help_lists_the_workloads_and_flags():
    r = _run("--help")
    assert r.returncode == 0
    for word in ("--workload", "--steps", "--warmup", "--gpus", "--cache-policy", "--versioned", "--event-every", "5mq4"):
        assert word in r.stdout
