"""Host-side half of the C ABI: the library loads, exports every symbol the
header declares, its size arithmetic is right and every argument error is
reported before any GPU call.  No GPU needed."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

from paper_1705_01626_amd import build as zvc_build
from paper_1705_01626_amd import zvc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    zvc_build.ensure_built()
    return zvc.load()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "zvc.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(zvc_[a-z_]+)\s*\(", header))
    assert declared == set(zvc.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_size_arithmetic():
    for n in (0, 1, 31, 32, 33, 4096, 4097, 205520896):
        G = (n + 31) // 32
        assert zvc.zvc_mask_bytes(n) == 4 * G
        assert zvc.zvc_max_compressed_bytes(n, 4) == 4 * G + 4 * n
        assert zvc.zvc_max_compressed_bytes(n, 2) == 4 * G + 2 * n
        assert zvc.zvc_workspace_bytes(n, 4) >= 256
        assert zvc.zvc_workspace_bytes(n, 4) % 8 == 0
    assert zvc.zvc_max_compressed_bytes(100, 3) == 0
    assert zvc.zvc_workspace_bytes(100, 8) == 0
    # workspace grows with n, and a 16-bit tensor never needs more than fp32
    assert zvc.zvc_workspace_bytes(1 << 28, 4) > zvc.zvc_workspace_bytes(1 << 20, 4)
    assert zvc.zvc_workspace_bytes(1 << 28, 2) <= zvc.zvc_workspace_bytes(1 << 28, 4)


def test_status_strings(lib):
    seen = set()
    for code, name in enumerate(zvc.STATUS_NAMES):
        s = zvc.status_string(code)
        assert s.startswith(name)
        seen.add(s)
    assert len(seen) == len(zvc.STATUS_NAMES)
    assert "unknown" in zvc.status_string(99)


def test_argument_errors_before_any_gpu_call(lib):
    """Fake but well-aligned addresses: validation must reject each call on the
    host, so nothing is launched (there is no GPU here)."""
    IN, OUT, WS, BY = 0x10000000, 0x20000000, 0x30000000, 0x40000000
    n, w = 1000, 4
    cap = zvc.zvc_max_compressed_bytes(n, w)
    wsb = zvc.zvc_workspace_bytes(n, w)
    c = lib.zvc_compress
    assert c(IN, n, 3, OUT, cap, BY, WS, wsb, None) == zvc.ZVC_E_WIDTH
    assert c(None, n, w, OUT, cap, BY, WS, wsb, None) == zvc.ZVC_E_ARG
    assert c(IN, n, w, None, cap, BY, WS, wsb, None) == zvc.ZVC_E_ARG
    assert c(IN, n, w, OUT, cap, None, WS, wsb, None) == zvc.ZVC_E_ARG
    assert c(IN + 2, n, w, OUT, cap, BY, WS, wsb, None) == zvc.ZVC_E_ALIGN
    assert c(IN, n, w, OUT + 2, cap, BY, WS, wsb, None) == zvc.ZVC_E_ALIGN
    assert c(IN, n, w, OUT, cap, BY + 4, WS, wsb, None) == zvc.ZVC_E_ALIGN
    assert c(IN, n, w, OUT, cap - 1, BY, WS, wsb, None) == zvc.ZVC_E_CAPACITY
    assert c(IN, n, w, IN + 400, cap, BY, WS, wsb, None) == zvc.ZVC_E_ARG  # overlap
    assert c(IN, n, w, OUT, cap, BY, None, wsb, None) == zvc.ZVC_E_ARG
    assert c(IN, n, w, OUT, cap, BY, WS + 64, wsb, None) == zvc.ZVC_E_ALIGN
    assert c(IN, n, w, OUT, cap, BY, WS, wsb - 1, None) == zvc.ZVC_E_WORKSPACE
    b = lib.zvc_compress_bounded
    masks = zvc.zvc_mask_bytes(n)
    assert b(IN, n, 3, 0, OUT, cap, BY, WS, wsb, None) == zvc.ZVC_E_WIDTH
    assert b(IN, n, w, 2, OUT, cap, BY, WS, wsb, None) == zvc.ZVC_E_ARG
    assert b(IN, n, w, 0, OUT, masks - 1, BY, WS, wsb, None) == zvc.ZVC_E_CAPACITY
    assert b(IN, n, w, 1, OUT + 2, masks, BY, WS, wsb, None) == zvc.ZVC_E_ALIGN
    assert b(IN, n, w, 0, IN + 4000 - masks + 4, masks, BY, WS, wsb, None) == zvc.ZVC_E_ARG  # overlap
    assert b(IN, n, w, 0, OUT, masks, BY, WS, wsb - 1, None) == zvc.ZVC_E_WORKSPACE
    d = lib.zvc_decompress
    assert d(OUT, cap, n, 5, IN, WS, wsb, None) == zvc.ZVC_E_WIDTH
    assert d(None, cap, n, w, IN, WS, wsb, None) == zvc.ZVC_E_ARG
    assert d(OUT, zvc.zvc_mask_bytes(n) - 1, n, w, IN, WS, wsb, None) == zvc.ZVC_E_CAPACITY
    assert d(OUT, cap, n, w, IN + 1, WS, wsb, None) == zvc.ZVC_E_ALIGN
    assert d(OUT, cap, n, w, OUT + 64, WS, wsb, None) == zvc.ZVC_E_ARG  # overlap
    assert d(OUT, cap, n, w, IN, WS, 8, None) == zvc.ZVC_E_WORKSPACE
    s = lib.zvc_compressed_size
    assert s(IN, n, 1, BY, WS, wsb, None) == zvc.ZVC_E_WIDTH
    assert s(IN, n, w, None, WS, wsb, None) == zvc.ZVC_E_ARG
    assert s(IN, n, w, BY, WS, 0, None) == zvc.ZVC_E_WORKSPACE
    o = lib.zvc_offload
    H = 0x50000000
    assert o(IN, n, 7, OUT, cap, H, cap, H + cap, WS, wsb, None, None) == zvc.ZVC_E_WIDTH
    assert o(IN, n, w, OUT, cap, H, cap - 4, H + cap, WS, wsb, None, None) == zvc.ZVC_E_CAPACITY
    assert o(IN, n, w, OUT, cap, H, cap, None, WS, wsb, None, None) == zvc.ZVC_E_ARG
    assert o(IN, n, w, OUT, cap - 4, H, cap, H + cap, WS, wsb, None, None) == zvc.ZVC_E_CAPACITY
    p = lib.zvc_prefetch
    assert p(H, cap, n, 3, OUT, cap, IN, WS, wsb, None, None) == zvc.ZVC_E_WIDTH
    assert p(H, zvc.zvc_mask_bytes(n) - 4, n, w, OUT, cap, IN, WS, wsb, None, None) == zvc.ZVC_E_CORRUPT
    assert p(H, cap + 4, n, w, OUT, cap + 4, IN, WS, wsb, None, None) == zvc.ZVC_E_CORRUPT
    assert p(H, cap, n, w, OUT, cap - 4, IN, WS, wsb, None, None) == zvc.ZVC_E_CAPACITY
    assert lib.zvc_workspace_init(None, 4096, None) == zvc.ZVC_E_ARG
    assert lib.zvc_workspace_init(WS, 100, None) == zvc.ZVC_E_WORKSPACE
    assert lib.zvc_workspace_init(WS + 8, 4096, None) == zvc.ZVC_E_ALIGN
    r = lib.zvc_reference_stream
    assert r(None, 64, OUT, 64, None) == zvc.ZVC_E_ARG
    assert r(IN, 64, None, 64, None) == zvc.ZVC_E_ARG
    assert r(IN + 4, 64, OUT, 64, None) == zvc.ZVC_E_ALIGN
    assert r(IN, 60, OUT, 64, None) == zvc.ZVC_E_ALIGN
    assert r(IN, 64, OUT, 72, None) == zvc.ZVC_E_ALIGN
    assert r(IN, 4096, IN + 1024, 4096, None) == zvc.ZVC_E_ARG  # overlap
    assert r(IN, 0, OUT, 0, None) == zvc.ZVC_OK                  # nothing to do, nothing launched
    q = lib.zvc_workspace_set_lookback_patience
    assert q(None, 5, None) == zvc.ZVC_E_ARG
    assert q(WS + 8, 5, None) == zvc.ZVC_E_ALIGN
    t = lib.zvc_compress_static
    assert t(IN, n, 3, OUT, cap, BY, None) == zvc.ZVC_E_WIDTH
    assert t(IN, (zvc.STATIC_MAX_BYTES // w) + 1, w, OUT, 1 << 40, BY, None) == zvc.ZVC_E_WORKSPACE
    wc = lib.zvc_window_compress
    OFF = 0x60000000
    assert wc(IN, n, w, 4096, OUT, cap, None, BY, WS, wsb, None) == zvc.ZVC_E_ARG
    assert wc(IN, n, w, 4096, OUT, cap, OFF + 4, BY, WS, wsb, None) == zvc.ZVC_E_ALIGN
    assert wc(IN, n, w, 5000, OUT, cap, OFF, BY, WS, wsb, None) == zvc.ZVC_E_ARG
    assert wc(IN, n, w, 4096, OUT, cap - 1, OFF, BY, WS, wsb, None) == zvc.ZVC_E_CAPACITY
    wd = lib.zvc_window_decompress
    assert wd(OUT, cap, OFF, n, w, 4096, 0, 2, IN, None) == zvc.ZVC_E_ARG          # one window only
    assert wd(OUT, cap, OFF, n, w, 1024, 3, 2, IN, None) == zvc.ZVC_E_ARG          # four windows of 1 KB
    assert wd(OUT, cap, OFF, n, w, 1024, 4, 0, IN, None) == zvc.ZVC_OK             # empty range at the end
    assert wd(OUT, cap, OFF, n, w, 100, 0, 1, IN, None) == zvc.ZVC_E_ARG
    assert wd(OUT, cap, OFF, n, 8, 4096, 0, 1, IN, None) == zvc.ZVC_E_WIDTH
    assert wd(OUT, cap, OFF + 4, n, w, 4096, 0, 1, IN, None) == zvc.ZVC_E_ALIGN
    assert wd(OUT, cap, OFF, n, w, 4096, 0, 1, OUT + 64, None) == zvc.ZVC_E_ARG    # overlap


def test_check_stream_on_host(oracle):
    """zvc_check_stream accepts exactly the streams whose size matches their
    masks.  Streams come from the oracle; the damage is done here."""
    rng = np.random.default_rng(2)
    for w in (2, 4):
        for n in (0, 1, 33, 1000, 4097):
            dtype = np.uint32 if w == 4 else np.uint16
            x = rng.integers(0, 3, size=n).astype(dtype)
            s = oracle.compress_stream(x, w)
            t = torch.from_numpy(np.concatenate([s, np.zeros(16, np.uint8)]))
            assert zvc.zvc_check_stream(t, s.size, n, w) == zvc.ZVC_OK
            if n:
                assert zvc.zvc_check_stream(t, s.size + w, n, w) == zvc.ZVC_E_CORRUPT
                assert zvc.zvc_check_stream(t, 4 * ((n + 31) // 32) - 1, n, w) == zvc.ZVC_E_CORRUPT
                t2 = t.clone()
                t2[0] ^= 1  # flip one presence bit: popcount no longer matches the size
                assert zvc.zvc_check_stream(t2, s.size, n, w) == zvc.ZVC_E_CORRUPT
            if n % 32:
                t3 = t.clone()
                G = (n + 31) // 32
                t3[4 * G - 1] |= 0x80  # a presence bit past n
                assert zvc.zvc_check_stream(t3, s.size, n, w) == zvc.ZVC_E_CORRUPT
    assert zvc.zvc_check_stream(torch.zeros(4, dtype=torch.uint8), 4, 32, 3) == zvc.ZVC_E_WIDTH


def test_window_check_stream_on_host(oracle):
    """zvc_window_check_stream accepts the oracle's windowed streams and tables and rejects
    damaged ones: a flipped presence bit, a shifted table entry, a wrong total, a bit past n."""
    rng = np.random.default_rng(3)
    for w in (2, 4):
      for window in (1024, 4096, 65536):
        per = zvc.zvc_window_elements(w, window)
        assert per == window // w
        for n in (0, 1, 33, per, per + 1, 5 * per + 77):
            dtype = np.uint32 if w == 4 else np.uint16
            x = rng.integers(0, 3, size=n).astype(dtype)
            s, offs = oracle.window_compress(x, w, per)
            assert zvc.zvc_window_count(n, w, window) == offs.size - 1
            t = torch.from_numpy(np.concatenate([s, np.zeros(16, np.uint8)]))
            o = torch.from_numpy(offs.astype(np.int64))
            assert zvc.zvc_window_check_stream(t, s.size, o, n, w, window) == zvc.ZVC_OK
            if n:
                t2 = t.clone()
                t2[0] ^= 1
                assert zvc.zvc_window_check_stream(t2, s.size, o, n, w, window) == zvc.ZVC_E_CORRUPT
                assert zvc.zvc_window_check_stream(t, s.size + w, o, n, w, window) == zvc.ZVC_E_CORRUPT
            if offs.size > 2:
                o2 = o.clone()
                o2[1] += w
                assert zvc.zvc_window_check_stream(t, s.size, o2, n, w, window) == zvc.ZVC_E_CORRUPT
                # a table made for another window size is not this stream's table
                if window < 65536:
                    assert zvc.zvc_window_check_stream(t, s.size, o, n, w, window * 2) == zvc.ZVC_E_CORRUPT
    # window sizes the library does not take
    for window in (0, 1000, 512, 3072, 131072):
        assert zvc.zvc_window_count(100, 4, window) == 0 and zvc.zvc_window_elements(4, window) == 0
        assert zvc.zvc_window_check_stream(torch.zeros(4, dtype=torch.uint8), 4,
                                           torch.zeros(2, dtype=torch.int64), 32, 4, window) == zvc.ZVC_E_ARG
    assert zvc.zvc_window_elements(3, 4096) == 0
    assert zvc.zvc_window_check_stream(torch.zeros(4, dtype=torch.uint8), 4,
                                       torch.zeros(2, dtype=torch.int64), 32, 3) == zvc.ZVC_E_WIDTH


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(zvc, "_lib", None)
    monkeypatch.setattr(zvc, "LIBRARY", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        zvc.load()


C_CLIENT = r"""
#include "zvc.h"
#include <stdio.h>
int main(void) {
    /* host-only entry points, called from plain C through the header's prototypes */
    if (zvc_mask_bytes(65) != 12) return 1;
    if (zvc_max_compressed_bytes(65, 2) != 12 + 130) return 2;
    if (zvc_workspace_bytes(1000, 4) == 0 || zvc_workspace_bytes(1000, 3) != 0) return 3;
    if (zvc_window_count(1025, 4, ZVC_WINDOW_PAPER_BYTES) != 2 || zvc_window_elements(2, 1024) != 512) return 4;
    unsigned int stream[3] = {0x5u, 7u, 9u};             /* one group of 3 elements: mask 101b, two values */
    if (zvc_check_stream(stream, 12, 3, 4) != ZVC_OK) return 5;
    if (zvc_check_stream(stream, 8, 3, 4) != ZVC_E_CORRUPT) return 6;
    if (zvc_compress(0, 10, 4, 0, 0, 0, 0, 0, 0) != ZVC_E_ARG) return 7;
    printf("%s\n", zvc_status_string(ZVC_E_WIDTH));
    return 0;
}
"""


def test_header_is_plain_c_and_links(lib, tmp_path):
    """include/zvc.h compiles as C11 with gcc and a C program links against the library."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "client.c"
    src.write_text(C_CLIENT)
    exe = tmp_path / "client"
    libdir = os.path.dirname(zvc.LIBRARY)
    cmd = ["gcc", "-std=c11", "-Wall", "-Werror=implicit-function-declaration", "-D__HIP_PLATFORM_AMD__",
           "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"), str(src), "-o", str(exe),
           "-L" + libdir, "-l:" + os.path.basename(zvc.LIBRARY), "-Wl,-rpath," + libdir]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    run = subprocess.run([str(exe)], capture_output=True, text=True)
    assert run.returncode == 0, (run.returncode, run.stdout, run.stderr)
    assert run.stdout.strip() != ""
