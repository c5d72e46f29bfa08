"""bench.py's command line on a machine without a GPU: what it refuses and what it offers."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_help_names_the_workloads_and_the_diagnostic_flag():
    r = run("--help")
    assert r.returncode == 0
    for word in ("--attn-config", "--copies-only", "--zero-inputs", "--cpu-rows"):
        assert word in r.stdout
