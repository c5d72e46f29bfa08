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


def test_the_product_path_fails_loudly_without_its_library(tmp_path):
    """No CPU fallback: with the shared library absent every entry point raises, naming the file to build."""
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "from paper_2407_00079_amd import binding as B\n"
        "B.LIB_PATH = %r\n"
        "try:\n"
        "    B.mc_prefill_attn_workspace_bytes(B.attn_params(8, 1, 128, 16, 64, 'bf16'), 1, 16)\n"
        "except RuntimeError as e:\n"
        "    print('raised:', e)\n"
        "else:\n"
        "    print('no error')\n" % (ROOT, str(tmp_path / "libmooncake_hip.so")))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    assert "raised:" in r.stdout and "is missing" in r.stdout and "no CPU fallback" in r.stdout


def test_the_package_does_not_touch_the_oracle():
    """The oracle is test infrastructure: nothing under the package imports, links or opens it."""
    pkg = os.path.join(ROOT, "paper_2407_00079_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath or "__pycache__" in dirpath:
            continue
        for name in files:
            if name.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, name), errors="replace").read()
                assert "mc_oracle" not in text and "import oracle" not in text and "from oracle" not in text, name
