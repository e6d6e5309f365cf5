"""bench.py's command line as the harness uses it (no GPU needed for what is checked here)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = run("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert p.returncode != 0
    assert "one GPU" in p.stderr
    assert p.stdout.strip() == ""


def test_help_lists_the_modes():
    p = run("--help")
    assert p.returncode == 0
    for word in ("--gpus", "--steps", "--warmup", "--workload", "--ceilings", "sweep", "opt66b_infer"):
        assert word in p.stdout
