"""bench.py command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], stdout=subprocess.PIPE,
                          stderr=subprocess.PIPE, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = run("--gpus", "2")
    assert p.returncode == 2
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_help_lists_the_workloads():
    p = run("--help")
    assert p.returncode == 0
    for word in ("--steps", "--warmup", "--config", "alignment sweep", "resource provisioning"):
        assert word in p.stdout
