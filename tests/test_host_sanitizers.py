"""Builds the host-only sources of the library with AddressSanitizer + UBSan (plain g++, no GPU code)
together with a randomised driver and runs it."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_under_asan_ubsan(tmp_path):
    exe = tmp_path / "host_fuzz"
    csrc = os.path.join(ROOT, "paper_2404_09336_amd", "csrc")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",   # the runtime is linked in: no ordering issue with preloaded libraries
           "-I" + os.path.join(ROOT, "include"), "-I" + csrc, os.path.join(ROOT, "tests", "host_fuzz.cpp"),
           os.path.join(csrc, "span_host.cpp"), "-o", str(exe)]
    subprocess.run(cmd, check=True)
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    sys.stdout.write(res.stdout[-2000:])
    assert res.returncode == 0 and "host_fuzz: ok" in res.stdout
