"""Compile the HIP library (csrc/*.hip -> libriver.so) for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "river.hip")
DEPS = [SRC, os.path.join(HERE, "csrc", "river_device.h"), os.path.join(HERE, "csrc", "river_prefill.h"),
        os.path.join(ROOT, "include", "river.h")]
LIB = os.path.join(HERE, "libriver.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
    # packed-fp32 instruction selection is switched off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-parameter",
]


def is_stale() -> bool:
    return (not os.path.exists(LIB)
            or any(os.path.getmtime(LIB) < os.path.getmtime(d) for d in DEPS))


TRACE_LIB = os.path.join(HERE, "libriver_trace.so")


def build(force: bool = True, trace: bool = False) -> str:
    """trace=True builds the diagnostics variant (per-barrier device timestamps)."""
    out = TRACE_LIB if trace else LIB
    if not force and not trace and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *(["-DRIVER_TRACE"] if trace else []),
           "-I", os.path.join(ROOT, "include"), "-o", out, SRC]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build())
