"""AddressSanitizer + UndefinedBehaviorSanitizer over the host-side code: the C ABI's argument validation
(csrc/flat_api.hip, flat_plan.hip and flat_probe_api.hip compiled as plain C++ against stub launchers) and the CPU oracle, driven by
tests/sanitize/host_check.cpp.  No GPU and no HIP runtime are involved."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_validation_code_and_oracle_are_clean_under_asan_and_ubsan():
    if shutil.which("g++") is None:
        pytest.skip("g++ not available")
    if not os.path.isdir("/opt/rocm/include/hip"):
        pytest.skip("HIP headers not available")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "host_check")
        cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
               "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-pthread", "-o", exe,
               "-x", "c++", os.path.join(ROOT, "paper_2107_06419_amd", "csrc", "flat_api.hip"),
               os.path.join(ROOT, "paper_2107_06419_amd", "csrc", "flat_plan.hip"),
               os.path.join(ROOT, "paper_2107_06419_amd", "csrc", "flat_probe_api.hip"),
               os.path.join(ROOT, "oracle", "flat_oracle.cpp"), os.path.join(ROOT, "tests", "sanitize", "host_check.cpp")]
        built = subprocess.run(cmd, capture_output=True, text=True)
        assert built.returncode == 0, built.stderr[-4000:]
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        env.pop("LD_PRELOAD", None)  # the sanitizer runtime has to come first in this one child process
        run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
        out = run.stdout + run.stderr
        assert run.returncode == 0, out[-4000:]
        assert "host checks passed" in out
        assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
