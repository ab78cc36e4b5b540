"""Builds the host side of libspin (tables, decomposition, tiling check, scheduler -- no GPU code)
together with a stress driver under AddressSanitizer + UndefinedBehaviorSanitizer and runs it."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not found")
def test_host_code_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_fuzz")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2503_15921_amd", "csrc"),
           os.path.join(ROOT, "tests", "native", "host_fuzz.cpp"),
           os.path.join(ROOT, "paper_2503_15921_amd", "csrc", "spin_host.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    r = subprocess.run([exe, "200"], capture_output=True, text=True, timeout=600, env=env)
    sys.stdout.write(r.stdout)
    sys.stderr.write(r.stderr[-4000:])
    assert r.returncode == 0
    assert "host fuzz ok" in r.stdout
