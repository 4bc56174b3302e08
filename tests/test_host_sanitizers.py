"""The host side of the library (descriptor validation, batch plan, bucketing programme) built with
AddressSanitizer and UBSan and driven with random segment tables.  CPU only, no HIP code involved."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2509_01193_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_under_asan_and_ubsan():
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "host_fuzz")
        cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC, os.path.join(ROOT, "tests", "host_fuzz.cpp"),
               os.path.join(CSRC, "plan.cpp"), os.path.join(CSRC, "bucketing.cpp"), "-o", exe]
        b = subprocess.run(cmd, capture_output=True, text=True)
        if b.returncode != 0 and "sanitize" in b.stderr:
            pytest.skip("sanitizer runtime not available: " + b.stderr[-200:])
        assert b.returncode == 0, b.stderr
        r = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                           env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
        assert r.returncode == 0 and "host fuzz ok" in r.stdout, r.stdout + r.stderr
