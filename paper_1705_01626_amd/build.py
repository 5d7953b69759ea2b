"""Compile the HIP library in-tree: csrc/zvc.hip -> paper_1705_01626_amd/libzvc.so.

Usage: python -m paper_1705_01626_amd.build
hipcc cross-compiles for gfx950, so this works on a machine without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SOURCE = os.path.join(PKG, "csrc", "zvc.hip")
LIBRARY = os.path.join(PKG, "libzvc.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def build(output: str = LIBRARY, extra=()) -> str:
    cmd = [HIPCC, *FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-o", output, SOURCE]
    subprocess.run(cmd, check=True)
    return output


def ensure_built() -> str:
    """Build only if nothing is built yet (or the source is newer)."""
    if (not os.path.exists(LIBRARY)
            or os.path.getmtime(LIBRARY) < os.path.getmtime(SOURCE)):
        build()
    return LIBRARY


if __name__ == "__main__":
    print(build(extra=sys.argv[1:]))
