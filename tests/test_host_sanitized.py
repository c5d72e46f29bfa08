"""Host code under AddressSanitizer and UBSan (CPU only).

* The planning / validation half of the library (csrc/host_plan.cpp, no HIP calls) is built with
  g++ -fsanitize=address,undefined together with tests/host_plan_driver.cpp.  Its self-test covers the
  rejection cases and the staging-slot state machine (two interleaved acquires never share a slot); the
  work lists it prints for the cases of test_host_plan.py must satisfy the same expectations and equal
  what the HIP library's mc_prefill_attn_plan returns.
* The oracle is built with the same sanitizers and its pins are run under them in a child process.
"""
import os
import subprocess
import sys

import pytest

from paper_2407_00079_amd import binding as B
from test_host_plan import CASES, expected

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2407_00079_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("host") / "host_plan_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", *SAN, "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", exe, os.path.join(ROOT, "tests", "host_plan_driver.cpp"), os.path.join(CSRC, "host_plan.cpp"), "-lpthread"]
    subprocess.run(cmd, check=True)
    return exe


def san_env():
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    return env


def test_rejections_and_slot_ring_under_sanitizers(driver):
    res = subprocess.run([driver, "selftest"], capture_output=True, text=True, env=san_env(), timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "selftest ok" in res.stdout and "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr


def ask(driver, requests):
    """requests: (Hq, Hkv, D, dtype, kv_splits, prefix, new) -> (status, items, suggested, list_bytes) each"""
    text = "".join(f"{Hq} {Hkv} {D} {dt} {s} {len(P)} " + " ".join(f"{p} {c}" for p, c in zip(P, C)) + "\n"
                   for Hq, Hkv, D, dt, s, P, C in requests)
    res = subprocess.run([driver, "plan"], input=text, capture_output=True, text=True, env=san_env(), timeout=300)
    assert res.returncode == 0 and res.stderr == "", res.stderr
    lines = res.stdout.split("\n")
    out, at = [], 0
    for _ in requests:
        st, n, sug, nbytes = (int(x) for x in lines[at].split())
        at += 1
        items = [tuple(int(x) for x in lines[at + i].split()) for i in range(max(n, 0))]
        at += max(n, 0)
        out.append((st, items, sug, nbytes))
    return out


def test_work_lists_under_sanitizers_equal_the_library(driver):
    if not os.path.exists(B.LIB_PATH):
        from paper_2407_00079_amd import build
        build.build()
    answers = ask(driver, [(Hq, Hkv, 128, 0, s, P, C) for Hq, Hkv, P, C, s in CASES])
    for (Hq, Hkv, P, C, s), (st, items, sug, nbytes) in zip(CASES, answers):
        assert st == B.MC_OK
        want = expected(Hq, Hkv, P, C, s)
        assert len(items) == len(set(items)) == len(want) and set(items) == set(want)
        p = B.attn_params(Hq, Hkv, 128, 16, 1 << 20, "bf16")
        assert items == B.mc_prefill_attn_plan(p, P, C, s)
        assert sug == B.mc_prefill_attn_suggest_kv_splits(p, P, C)
        assert nbytes >= 16 * len(items) + 16 * len(P)


def test_rejections_through_the_driver(driver):
    big = 2 ** 31 - 8
    answers = ask(driver, [(64, 7, 128, 0, 0, [10], [10]), (64, 8, 96, 0, 0, [10], [10]), (64, 8, 128, 5, 0, [10], [10]),
                           (64, 8, 128, 0, 0, [-1], [10]), (64, 8, 128, 0, 0, [10], [-2]), (64, 8, 128, 0, 300, [10], [10]),
                           (64, 8, 128, 0, 0, [big], [16]), (4, 1, 64, 1, 0, [256], [128]), (64, 8, 128, 0, 0, [], [])])
    sts = [a[0] for a in answers]
    assert sts == [B.MC_ERR_SHAPE, B.MC_ERR_UNSUPPORTED, B.MC_ERR_UNSUPPORTED, B.MC_ERR_SHAPE, B.MC_ERR_SHAPE,
                   B.MC_ERR_SHAPE, B.MC_ERR_RANGE, B.MC_OK, B.MC_OK]
    assert [a[2] for a in answers[:5]] == [0] * 5              # the slice suggestion refuses the same arguments
    assert len(answers[7][1]) == 2 and answers[8][1] == []     # configuration 1: 512 stacked rows, one KV head


def test_oracle_pins_under_sanitizers():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no AddressSanitizer runtime beside gcc")
    env = san_env()
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0"     # the interpreter's own allocations are not ours
    env["MC_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    files = ["test_oracle_attn.py", "test_oracle_pack.py", "test_oracle_append.py", "test_oracle_merge.py",
             "test_oracle_prefix.py"]
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          *[os.path.join(ROOT, "tests", f) for f in files]],
                         capture_output=True, text=True, env=env, cwd=ROOT, timeout=900)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
    assert os.path.exists(os.path.join(ROOT, "oracle", "libmc_oracle_san.so"))
