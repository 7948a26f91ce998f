"""Builds libharris.so for gfx950 with hipcc (cross-compiles without a GPU).

Every source file is compiled to an object of its own, all at once, and the objects are linked
into paper_2212_12035_amd/libharris.so; the objects live in a build folder beside it.
"""
from __future__ import annotations

import os
import subprocess
import sys

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
CSRC = os.path.join(_PKG, "csrc")
LIB = os.path.join(_PKG, "libharris.so")
BUILD_DIR = os.path.join(_PKG, "_build")

SOURCES = ("harris_tiles_f32.hip", "harris_tiles_u8.hip", "harris_bands.hip", "harris_grouped.hip", "harris_copy.hip",
           "harris_launch.cpp", "harris_api.cpp")
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # the compiler must not form packed-FP32 instructions on its own
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(_ROOT, "include"), "-I" + CSRC,
]


def build_library() -> str:
    """Compile and link the library; returns its path.  Raises RuntimeError with the compiler's output on failure."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(BUILD_DIR, exist_ok=True)
    jobs = []
    for name in SOURCES:
        obj = os.path.join(BUILD_DIR, os.path.splitext(name)[0] + ".o")
        cmd = [hipcc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, name), "-o", obj]
        jobs.append((name, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = []
    for name, obj, proc in jobs:
        out, _ = proc.communicate()
        if proc.returncode != 0:
            failed.append("%s:\n%s" % (name, out))
    if failed:
        raise RuntimeError("hipcc failed building libharris.so\n" + "\n".join(failed))
    tmp = LIB + ".tmp.%d" % os.getpid()
    link = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[obj for _, obj, _ in jobs], "-o", tmp],
                          capture_output=True, text=True)
    if link.returncode != 0:
        raise RuntimeError("hipcc failed linking libharris.so\n" + link.stdout + link.stderr)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print("built", build_library())
    sys.exit(0)
