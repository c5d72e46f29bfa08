"""The product path has no CPU fallback and no tie to the oracle."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


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
