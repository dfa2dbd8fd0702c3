"""Builds the C-ABI library (csrc/ -> liboserve.so, in-tree) with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liboserve.so")
SOURCES = ["kernels.hip", "prefill.hip", "migrate.hip", "static_scratch.hip", "mixed.hip", "api.cpp", "api_prefill.cpp", "api_migrate.cpp", "api_mixed.cpp", "plan.cpp", "prefill_plan.cpp", "planner.cpp"]
HEADERS = ["kernels.h", "plan.h", "host_util.h", "decode_launch.h", "prefill_plan.h", "decode_body.h", "prefill_body.h", "launch_util.h", os.path.join(ROOT, "include", "oserve.h")]


def hipcc_command(out: str = LIB) -> list:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
            "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
            # packed-fp32 instructions are kept out of all device code on the test machines
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-command-line-argument",
            "-o", out] + [os.path.join(CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + [h if os.path.isabs(h) else os.path.join(CSRC, h) for h in HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(force: bool = True) -> str:
    if force or is_stale():
        proc = subprocess.run(hipcc_command(), stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        # the host pass warns that it does not know the packed-fp32 feature: harmless
        noise = "is not a recognized feature for this target"
        out = "\n".join(l for l in proc.stdout.splitlines() if noise not in l)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)
        if out.strip():
            print(out)
    return LIB


if __name__ == "__main__":
    print(build_library(True))
