"""The host-side C/C++ of both sides under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only):
the library's preparation (bda_prepare.cpp) and the oracle's loops (oracle/bd_project.c) are
compiled with gcc's sanitizers together with a small driver that reaches every mode, side, storage
type, window position and error path, and the program must exit cleanly."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="needs gcc / g++")
def test_prepare_and_oracle_loops_under_asan_ubsan(tmp_path):
    obj = str(tmp_path / "bd_project.o")
    exe = str(tmp_path / "host_sanitize")
    subprocess.run(["gcc", "-std=c11", "-fopenmp", *SAN, "-c", os.path.join(ROOT, "oracle", "bd_project.c"), "-o", obj],
                   check=True)
    subprocess.run(["g++", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"),
                    "-I", os.path.join(ROOT, "paper_2510_01718_amd", "csrc"),
                    os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"),
                    os.path.join(ROOT, "paper_2510_01718_amd", "csrc", "bda_prepare.cpp"), obj,
                    "-static-libasan", "-static-libubsan",      # static runtimes: no library-order requirement at start-up
                    "-fopenmp", "-lpthread", "-o", exe], check=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    proc = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert proc.returncode == 0, proc.stdout[-4000:]
    assert "all checks passed" in proc.stdout
