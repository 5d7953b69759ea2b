"""The oracle and the host half of the C ABI under AddressSanitizer and UBSan:
both are built instrumented into a temporary directory and their CPU test files
are run against those builds in a child process (the sanitizer runtime has to be
loaded before Python starts).  No GPU needed."""
import os
import subprocess
import sys

import pytest

from oracle import build as oracle_build
from paper_1705_01626_amd import build as zvc_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# leaks of the interpreter itself are not ours; the harness preloads a library of its own before the runtime
ASAN_OPTIONS = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:halt_on_error=1"


def run_child(code, preload, extra_env):
    env = dict(os.environ)
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = ASAN_OPTIONS
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra_env)
    return subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True,
                          timeout=900)


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    lib = oracle_build.build(output=str(tmp_path / "libzvc_ref_san.so"), sanitize=True)
    code = ("import sys, pytest; sys.exit(pytest.main(['-q', '-x', '-p', 'no:cacheprovider', "
            "'tests/test_oracle.py', 'tests/test_oracle_relu.py', 'tests/test_oracle_window.py', "
            "'tests/test_rle_layout.py', '-m', 'not gpu']))")
    done = run_child(code, oracle_build.asan_runtime(), {"ZVC_REF_LIBRARY": lib})
    assert done.returncode == 0, done.stdout[-3000:] + done.stderr[-3000:]
    assert "passed" in done.stdout
    assert "ERROR: AddressSanitizer" not in done.stderr and "runtime error" not in done.stderr


def test_host_abi_under_asan_and_ubsan(tmp_path):
    """The library's host code (argument checks, size arithmetic, stream checks) instrumented;
    the device code is compiled as usual."""
    lib = str(tmp_path / "libzvc_san.so")
    zvc_build.build(output=lib, extra=["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
                                      "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"])
    runtime = subprocess.run([zvc_build.HIPCC, "--print-file-name=libclang_rt.asan-x86_64.so"], check=True,
                             capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("the HIP compiler's AddressSanitizer runtime was not found")
    code = ("import sys, pytest\n"
            "import paper_1705_01626_amd.zvc as z, paper_1705_01626_amd.build as b\n"
            "z.LIBRARY = %r\n"
            "b.ensure_built = lambda: %r\n"
            # the C client of the header test links with plain gcc, which an instrumented library does not allow
            "sys.exit(pytest.main(['-q', '-x', '-p', 'no:cacheprovider', 'tests/test_host_abi.py', "
            "'--deselect', 'tests/test_host_abi.py::test_header_is_plain_c_and_links']))\n" % (lib, lib))
    done = run_child(code, runtime, {})
    assert done.returncode == 0, done.stdout[-3000:] + done.stderr[-3000:]
    assert "passed" in done.stdout
    assert "ERROR: AddressSanitizer" not in done.stderr and "runtime error" not in done.stderr
