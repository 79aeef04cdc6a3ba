"""Compile the HIP library (csrc/*.hip -> libriver.so) for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "river.hip")
DEPS = [SRC, os.path.join(HERE, "csrc", "river_device.h"), os.path.join(ROOT, "include", "river.h")]
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


def build(force: bool = True) -> str:
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
