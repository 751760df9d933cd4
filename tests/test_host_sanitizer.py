"""Host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.

The entry points' own work (validation, segment and run tables, workspace layout, selection and weight vectors) is
compiled from the library's sources by the plain host C++ compiler against a stand-in for the HIP runtime header,
linked with recording stubs in place of the kernel launchers and a driver of checks (tests/host_sanitizer/), and
run as an ordinary CPU program.  No GPU code is built or run here."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HS = os.path.join(ROOT, "tests", "host_sanitizer")
CSRC = os.path.join(ROOT, "paper_2505_16710_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_host_entry_points_are_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitizer_run")
    flags = ["-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
             "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", "-Wall",
             "-I", HS, "-I", os.path.join(ROOT, "include"), "-I", CSRC]      # HS first: its hip/hip_runtime.h wins
    srcs = ["-x", "c++", os.path.join(CSRC, "seco_api.hip"), os.path.join(CSRC, "seco_select.cpp"),
            os.path.join(HS, "stub_launch.cpp"), os.path.join(HS, "driver.cpp")]
    r = subprocess.run(["g++", *flags, *srcs, "-o", exe, "-lpthread"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "all checks passed" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
