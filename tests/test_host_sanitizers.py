"""The library's host-only sources (share planning, bucket layout + tile table,
sampler partition) built with AddressSanitizer and UBSan and driven with random
inputs.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_10183_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_under_sanitizers(tmp_path):
    exe = str(tmp_path / "fuzz_host")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           "-ffp-contract=off", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host", "fuzz_host.cpp"), os.path.join(CSRC, "kt_plan.cpp"),
           os.path.join(CSRC, "kt_sampler.cpp"), "-o", exe]
    subprocess.check_call(cmd)
    out = subprocess.run([exe, "4000"], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stdout + out.stderr
    assert out.stdout.startswith("ok"), out.stdout + out.stderr
