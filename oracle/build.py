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
    """Build `source` into the shared library `output` and return its path.  With
    `sanitize` the library is instrumented with AddressSanitizer and UBSan (a process
    that loads it needs libasan preloaded: `asan_runtime()`)."""
    cmd = ["g++", "-std=c++17", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC"]
    if sanitize:
        cmd += ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    cmd += ["-o", output, source]
    subprocess.run(cmd, check=True)
    return output


def asan_runtime() -> str:
    """Path of the host compiler's AddressSanitizer runtime (to preload)."""
    return subprocess.run(["g++", "-print-file-name=libasan.so"], check=True, capture_output=True,
                          text=True).stdout.strip()


def ensure_built() -> str:
    """Build the oracle if the library is missing or older than its source.  ZVC_REF_LIBRARY
    names another build of the same source to use instead (the sanitizer test's)."""
    override = os.environ.get("ZVC_REF_LIBRARY")
    if override:
        return override
    if (not os.path.exists(LIBRARY)
            or os.path.getmtime(LIBRARY) < os.path.getmtime(SOURCE)):
        build()
    return LIBRARY


if __name__ == "__main__":
    print(build(sanitize="--sanitize" in sys.argv))
