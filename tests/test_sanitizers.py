"""AddressSanitizer + UndefinedBehaviorSanitizer build of the library's host-only code (split planner, prefill work
list, switch and assignment planners) and of the C++ oracle, driven over seeded random inputs (CPU only)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2602_12151_amd", "csrc")


def test_host_code_and_oracle_under_asan_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "host_fuzz")
    sources = [os.path.join(ROOT, "tests", "sanitize", "host_fuzz.cpp"),
               os.path.join(CSRC, "plan.cpp"), os.path.join(CSRC, "prefill_plan.cpp"), os.path.join(CSRC, "planner.cpp"),
               os.path.join(ROOT, "oracle", "paged_attention_oracle.cpp")]
    # kernels.h pulls in the HIP runtime's declarations (types only; nothing of the runtime is linked)
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-static-libasan", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-ffp-contract=off", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-I/opt/rocm/include",
           "-o", exe] + sources
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    if build.returncode != 0 and "sanitizer" in build.stdout.lower() and "cannot find" in build.stdout.lower():
        pytest.skip("sanitizer runtime not installed")
    assert build.returncode == 0, build.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe, "1500"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600, env=env)
    assert run.returncode == 0, run.stdout[-4000:]
    assert run.stdout.strip().endswith("planners") and "ok:" in run.stdout
