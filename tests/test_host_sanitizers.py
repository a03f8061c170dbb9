"""The library's host-only code (index maps, failover target, load-balancer arithmetic, the
buffer-overlap rules every GPU entry point applies before it launches anything) under
AddressSanitizer and UBSan, CPU only: tests/host_sanitize_driver.cpp is built with g++ and run."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_asan_and_ubsan():
    csrc = os.path.join(ROOT, "paper_2405_17870_amd", "csrc")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "host_sanitize")
        cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
               "-static-libasan", "-static-libubsan",
               "-I", os.path.join(ROOT, "include"), "-I", csrc,
               os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"),
               os.path.join(csrc, "nz_index.cpp"), os.path.join(csrc, "nz_balance.cpp"),
               os.path.join(csrc, "nz_validate.cpp"), os.path.join(csrc, "nz_placement.cpp"), "-o", exe]
        subprocess.run(cmd, check=True)
        r = subprocess.run([exe], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        assert "host sanitizer run ok" in r.stdout
