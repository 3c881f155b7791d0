"""The host selector (integer dynamic program of Section 6) under AddressSanitizer and UBSan: a few thousand random
and adversarial inputs; every returned mask must reproduce its own predicted time under the time model."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_selector_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "fuzz_select")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2312_14227_amd", "csrc"),
           "-o", exe, os.path.join(ROOT, "tests", "host", "fuzz_select.cpp")]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "runs 3000" in r.stdout and "mismatch" not in r.stdout, r.stdout
