"""ctypes binding of the C++ ZVC oracle (oracle/zvc_ref.cpp).

TEST INFRASTRUCTURE ONLY: marshals numpy buffers into the oracle's extern "C"
functions.  It holds none of the method's arithmetic and imports nothing from
the GPU package.
"""
from __future__ import annotations

import ctypes
from typing import Optional, Tuple

import numpy as np

from . import build as _build

_U64 = ctypes.c_uint64
_BAD = (1 << 64) - 1
_lib_cache = {}


def load(path: Optional[str] = None) -> ctypes.CDLL:
    """Load (building first if needed) the oracle library and set signatures."""
    path = path or _build.ensure_built()
    if path in _lib_cache:
        return _lib_cache[path]
    lib = ctypes.CDLL(path)
    vp, ip = ctypes.c_void_p, ctypes.c_int
    lib.zvc_ref_groups.restype = _U64
    lib.zvc_ref_groups.argtypes = [_U64]
    lib.zvc_ref_compress.restype = _U64
    lib.zvc_ref_compress.argtypes = [vp, _U64, ip, vp, vp]
    lib.zvc_ref_compressed_bytes.restype = _U64
    lib.zvc_ref_compressed_bytes.argtypes = [_U64, ip, _U64]
    lib.zvc_ref_compress_stream.restype = _U64
    lib.zvc_ref_compress_stream.argtypes = [vp, _U64, ip, vp]
    lib.zvc_ref_decompress.restype = _U64
    lib.zvc_ref_decompress.argtypes = [vp, vp, _U64, ip, vp]
    lib.zvc_ref_decompress_stream.restype = _U64
    lib.zvc_ref_decompress_stream.argtypes = [vp, _U64, ip, vp]
    lib.zvc_ref_count_nonzero.restype = _U64
    lib.zvc_ref_count_nonzero.argtypes = [vp, _U64, ip]
    if hasattr(lib, "zvc_ref_relu"):   # absent from mutated copies built before it existed
        lib.zvc_ref_relu.restype = ip
        lib.zvc_ref_relu.argtypes = [vp, _U64, ip, vp]
        lib.zvc_ref_relu_compress_stream.restype = _U64
        lib.zvc_ref_relu_compress_stream.argtypes = [vp, _U64, ip, vp]
    if hasattr(lib, "zvc_ref_window_compress"):
        lib.zvc_ref_window_count.restype = _U64
        lib.zvc_ref_window_count.argtypes = [_U64, _U64]
        lib.zvc_ref_window_compress.restype = _U64
        lib.zvc_ref_window_compress.argtypes = [vp, _U64, ip, _U64, vp, vp]
        lib.zvc_ref_window_decompress.restype = _U64
        lib.zvc_ref_window_decompress.argtypes = [vp, vp, _U64, ip, _U64, _U64, _U64, vp]
    _lib_cache[path] = lib
    return lib


def _as_bytes(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    return a.reshape(-1).view(np.uint8)


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def groups(n: int, lib=None) -> int:
    return int((lib or load()).zvc_ref_groups(n))


def compressed_bytes(n: int, w: int, nnz: int, lib=None) -> int:
    return int((lib or load()).zvc_ref_compressed_bytes(n, w, nnz))


def compress(x: np.ndarray, w: int, lib=None) -> Tuple[np.ndarray, np.ndarray, int]:
    """Encode the raw bytes of `x` as n = x.nbytes // w elements.

    Returns (masks uint32[G], values uint8[w * nnz], nnz).
    """
    lib = lib or load()
    raw = _as_bytes(x)
    n = raw.size // w
    masks = np.zeros(groups(n, lib), dtype=np.uint32)
    values = np.zeros(max(n * w, 1), dtype=np.uint8)
    nnz = lib.zvc_ref_compress(_ptr(raw), n, w, _ptr(masks), _ptr(values))
    if nnz == _BAD:
        raise ValueError("unsupported element width %r" % (w,))
    return masks, values[: nnz * w].copy(), int(nnz)


def compress_stream(x: np.ndarray, w: int, lib=None) -> np.ndarray:
    """Encode into the serialised [masks][values] byte stream (exact length)."""
    lib = lib or load()
    raw = _as_bytes(x)
    n = raw.size // w
    out = np.zeros(4 * groups(n, lib) + n * w + 1, dtype=np.uint8)
    used = lib.zvc_ref_compress_stream(_ptr(raw), n, w, _ptr(out))
    if used == _BAD:
        raise ValueError("unsupported element width %r" % (w,))
    return out[:used].copy()


def decompress(masks: np.ndarray, values: np.ndarray, n: int, w: int, lib=None) -> np.ndarray:
    """Decode to a uint8 array of n * w bytes."""
    lib = lib or load()
    masks = np.ascontiguousarray(masks, dtype=np.uint32)
    vals = _as_bytes(values) if values.size else np.zeros(1, dtype=np.uint8)
    out = np.full(max(n * w, 1), 0xAB, dtype=np.uint8)
    used = lib.zvc_ref_decompress(_ptr(masks), _ptr(vals), n, w, _ptr(out))
    if used == _BAD:
        raise ValueError("unsupported element width %r" % (w,))
    return out[: n * w]


def decompress_stream(stream: np.ndarray, n: int, w: int, lib=None) -> np.ndarray:
    lib = lib or load()
    comp = _as_bytes(stream) if stream.size else np.zeros(1, dtype=np.uint8)
    out = np.full(max(n * w, 1), 0xAB, dtype=np.uint8)
    used = lib.zvc_ref_decompress_stream(_ptr(comp), n, w, _ptr(out))
    if used == _BAD:
        raise ValueError("unsupported element width %r" % (w,))
    return out[: n * w]


def count_nonzero(x: np.ndarray, w: int, lib=None) -> int:
    lib = lib or load()
    raw = _as_bytes(x)
    return int(lib.zvc_ref_count_nonzero(_ptr(raw), raw.size // w, w))


def relu(x: np.ndarray, w: int, lib=None) -> np.ndarray:
    """ReLU of the raw bytes of `x` taken as w-byte sign-magnitude floats; uint8[n * w]."""
    lib = lib or load()
    raw = _as_bytes(x)
    n = raw.size // w
    out = np.full(max(n * w, 1), 0xAB, dtype=np.uint8)
    if lib.zvc_ref_relu(_ptr(raw), n, w, _ptr(out)) != 0:
        raise ValueError("unsupported element width %r" % (w,))
    return out[: n * w]


def relu_compress_stream(x: np.ndarray, w: int, lib=None) -> np.ndarray:
    """The [masks][values] stream of ReLU(x) (fused ReLU + ZVC)."""
    lib = lib or load()
    raw = _as_bytes(x)
    n = raw.size // w
    out = np.zeros(4 * groups(n, lib) + n * w + 1, dtype=np.uint8)
    used = lib.zvc_ref_relu_compress_stream(_ptr(raw), n, w, _ptr(out))
    if used == _BAD:
        raise ValueError("unsupported element width %r" % (w,))
    return out[:used].copy()


def window_count(n: int, window_elems: int, lib=None) -> int:
    return int((lib or load()).zvc_ref_window_count(n, window_elems))


def window_compress(x: np.ndarray, w: int, window_elems: int, lib=None) -> Tuple[np.ndarray, np.ndarray]:
    """Paper-order windowed stream of the raw bytes of `x`.

    Returns (stream uint8[bytes], offsets uint64[windows + 1])."""
    lib = lib or load()
    raw = _as_bytes(x)
    n = raw.size // w
    out = np.zeros(4 * groups(n, lib) + n * w + 1, dtype=np.uint8)
    windows = window_count(n, window_elems, lib) if window_elems else 0
    offsets = np.zeros(windows + 1, dtype=np.uint64)
    used = lib.zvc_ref_window_compress(_ptr(raw), n, w, window_elems, _ptr(out), _ptr(offsets))
    if used == _BAD:
        raise ValueError("unsupported width %r or window %r" % (w, window_elems))
    return out[:used].copy(), offsets


def window_decompress(stream: np.ndarray, offsets: np.ndarray, n: int, w: int, window_elems: int,
                      first_window: int, num_windows: int, lib=None) -> np.ndarray:
    """Elements of windows [first_window, first_window + num_windows) as uint8 bytes."""
    lib = lib or load()
    comp = _as_bytes(stream) if stream.size else np.zeros(1, dtype=np.uint8)
    offs = np.ascontiguousarray(offsets, dtype=np.uint64)
    elems = max(0, min(n, (first_window + num_windows) * window_elems) - first_window * window_elems)
    out = np.full(max(elems * w, 1), 0xAB, dtype=np.uint8)
    got = lib.zvc_ref_window_decompress(_ptr(comp), _ptr(offs), n, w, window_elems, first_window,
                                        num_windows, _ptr(out))
    if got == _BAD:
        raise ValueError("bad window arguments")
    assert got == elems
    return out[: elems * w]
