"""Host code under AddressSanitizer + UBSan (CPU only): the library's plan builder and the oracle,
each driven by a small randomised program with exact-size heap buffers."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def _build_and_run(tmp_path, compiler, sources, includes, extra=()):
    exe = str(tmp_path / "driver")
    cmd = [compiler, *SAN, *extra, *[f"-I{i}" for i in includes], *sources, "-o", exe, "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.startswith("ok"), res.stdout + res.stderr


def test_plan_builder_under_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2412_15411_amd", "csrc")
    _build_and_run(tmp_path, "g++", [os.path.join(ROOT, "tests", "sanitize", "plan_driver.cpp"), os.path.join(csrc, "plan.cpp")],
                   [os.path.join(ROOT, "include"), csrc], extra=["-std=c++17"])


def test_oracle_under_sanitizers(tmp_path):
    odir = os.path.join(ROOT, "oracle")
    _build_and_run(tmp_path, "gcc", [os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), os.path.join(odir, "moev_oracle.c")],
                   [odir], extra=["-std=c99", "-ffp-contract=off"])
