"""Compile the C++ oracle into oracle/libzvc_ref.so with the host compiler.

Test infrastructure only.  Usage: python -m oracle.build [--sanitize]
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(HERE, "zvc_ref.cpp")
LIBRARY = os.path.join(HERE, "libzvc_ref.so")


def build(output: str = LIBRARY, source: str = SOURCE, sanitize: bool = False) -> str:
    """Build `source` into the shared library `output` and return its path."""
    cmd = ["g++", "-std=c++17", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC"]
    if sanitize:
        cmd += ["-fsanitize=undefined", "-fno-sanitize-recover=all"]
    cmd += ["-o", output, source]
    subprocess.run(cmd, check=True)
    return output


def ensure_built() -> str:
    """Build the oracle if the library is missing or older than its source."""
    if (not os.path.exists(LIBRARY)
            or os.path.getmtime(LIBRARY) < os.path.getmtime(SOURCE)):
        build()
    return LIBRARY


if __name__ == "__main__":
    print(build(sanitize="--sanitize" in sys.argv))
