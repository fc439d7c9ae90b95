"""Host code under sanitizers (CPU only): the pool logic is compiled with
AddressSanitizer and UBSan and driven through a long random trace; the header
is compiled as plain C99."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_22416_amd", "csrc")
NATIVE = os.path.join(ROOT, "tests", "native")


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_pool_logic_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "pool_state_fuzz")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan",
           "-I", CSRC, os.path.join(NATIVE, "pool_state_fuzz.cpp"), os.path.join(CSRC, "pool_state.cpp"),
           "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    for seed in ("1", "2"):
        res = subprocess.run([exe, seed], capture_output=True, text=True, timeout=300)
        assert res.returncode == 0, res.stdout + res.stderr
        assert res.stdout.startswith("ok"), res.stdout
        assert "migrations=0" not in res.stdout and "rebalances=0" not in res.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no host compiler")
def test_header_compiles_as_c99(tmp_path):
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
           "-c", os.path.join(NATIVE, "header_is_c.c"), "-o", str(tmp_path / "h.o")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
