"""ctypes binding of libzvc.so (C ABI in include/zvc.h).

Argument marshalling only: torch tensors supply device memory and streams, the
library's HIP kernels do all the work.  There is no CPU fallback: if the
library is missing, `load()` raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIBRARY = os.path.join(_PKG, "libzvc.so")

STATUS_NAMES = ("ZVC_OK", "ZVC_E_ARG", "ZVC_E_WIDTH", "ZVC_E_CAPACITY", "ZVC_E_WORKSPACE",
                "ZVC_E_ALIGN", "ZVC_E_HIP", "ZVC_E_CORRUPT")
(ZVC_OK, ZVC_E_ARG, ZVC_E_WIDTH, ZVC_E_CAPACITY, ZVC_E_WORKSPACE, ZVC_E_ALIGN, ZVC_E_HIP,
 ZVC_E_CORRUPT) = range(8)

# window sizes of the windowed stream (ZVC_WINDOW_* of include/zvc.h): powers of two in between
WINDOW_MIN_BYTES, WINDOW_PAPER_BYTES, WINDOW_MAX_BYTES = 1024, 4096, 65536

# every symbol include/zvc.h declares
EXPORTS = ("zvc_status_string", "zvc_mask_bytes", "zvc_max_compressed_bytes",
           "zvc_workspace_bytes", "zvc_check_stream", "zvc_workspace_init",
           "zvc_compressed_size", "zvc_compress", "zvc_decompress", "zvc_offload",
           "zvc_prefetch", "zvc_workspace_set_lookback_patience", "zvc_workspace_self_help_count",
           "zvc_relu_compress", "zvc_relu_offload", "zvc_window_count", "zvc_window_elements",
           "zvc_window_check_stream",
           "zvc_window_compress", "zvc_window_decompress", "zvc_compress_bounded",
           "zvc_compress_static", "zvc_reference_stream")

_lib = None


class ZvcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, status_string(status)))


def load() -> ctypes.CDLL:
    """Load the built library (paper_1705_01626_amd/libzvc.so) and declare signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIBRARY):
        raise ImportError(
            "%s is not built: run `python -m paper_1705_01626_amd.build` (there is no CPU "
            "fallback)" % LIBRARY)
    lib = ctypes.CDLL(LIBRARY)
    vp, sz, ci, u64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_uint64
    lib.zvc_status_string.restype = ctypes.c_char_p
    lib.zvc_status_string.argtypes = [ci]
    lib.zvc_mask_bytes.restype = sz
    lib.zvc_mask_bytes.argtypes = [sz]
    lib.zvc_max_compressed_bytes.restype = sz
    lib.zvc_max_compressed_bytes.argtypes = [sz, ci]
    lib.zvc_workspace_bytes.restype = sz
    lib.zvc_workspace_bytes.argtypes = [sz, ci]
    lib.zvc_check_stream.restype = ci
    lib.zvc_check_stream.argtypes = [vp, u64, sz, ci]
    lib.zvc_workspace_init.restype = ci
    lib.zvc_workspace_init.argtypes = [vp, sz, vp]
    lib.zvc_compressed_size.restype = ci
    lib.zvc_compressed_size.argtypes = [vp, sz, ci, vp, vp, sz, vp]
    lib.zvc_compress.restype = ci
    lib.zvc_compress.argtypes = [vp, sz, ci, vp, sz, vp, vp, sz, vp]
    lib.zvc_compress_static.restype = ci
    lib.zvc_compress_static.argtypes = [vp, sz, ci, vp, sz, vp, vp]
    lib.zvc_window_count.restype = sz
    lib.zvc_window_count.argtypes = [sz, ci, sz]
    lib.zvc_window_elements.restype = sz
    lib.zvc_window_elements.argtypes = [ci, sz]
    lib.zvc_window_check_stream.restype = ci
    lib.zvc_window_check_stream.argtypes = [vp, u64, vp, sz, ci, sz]
    lib.zvc_window_compress.restype = ci
    lib.zvc_window_compress.argtypes = [vp, sz, ci, sz, vp, sz, vp, vp, vp, sz, vp]
    lib.zvc_window_decompress.restype = ci
    lib.zvc_window_decompress.argtypes = [vp, sz, vp, sz, ci, sz, sz, sz, vp, vp]
    lib.zvc_relu_compress.restype = ci
    lib.zvc_relu_compress.argtypes = [vp, sz, ci, vp, sz, vp, vp, sz, vp]
    lib.zvc_compress_bounded.restype = ci
    lib.zvc_compress_bounded.argtypes = [vp, sz, ci, ci, vp, sz, vp, vp, sz, vp]
    lib.zvc_decompress.restype = ci
    lib.zvc_decompress.argtypes = [vp, sz, sz, ci, vp, vp, sz, vp]
    lib.zvc_offload.restype = ci
    lib.zvc_offload.argtypes = [vp, sz, ci, vp, sz, vp, sz, vp, vp, sz, vp, vp]
    lib.zvc_relu_offload.restype = ci
    lib.zvc_relu_offload.argtypes = [vp, sz, ci, vp, sz, vp, sz, vp, vp, sz, vp, vp]
    lib.zvc_prefetch.restype = ci
    lib.zvc_prefetch.argtypes = [vp, u64, sz, ci, vp, sz, vp, vp, sz, vp, vp]
    lib.zvc_workspace_set_lookback_patience.restype = ci
    lib.zvc_workspace_set_lookback_patience.argtypes = [vp, ctypes.c_uint, vp]
    lib.zvc_reference_stream.restype = ci
    lib.zvc_reference_stream.argtypes = [vp, sz, vp, sz, vp]
    lib.zvc_workspace_self_help_count.restype = ci
    lib.zvc_workspace_self_help_count.argtypes = [vp, vp]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().zvc_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != ZVC_OK:
        raise ZvcError(status, where)


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def element_width(t: torch.Tensor) -> int:
    return t.element_size()


# ---- host arithmetic ---------------------------------------------------------
def zvc_mask_bytes(n: int) -> int:
    return int(load().zvc_mask_bytes(n))


def zvc_max_compressed_bytes(n: int, w: int) -> int:
    return int(load().zvc_max_compressed_bytes(n, w))


def zvc_workspace_bytes(n: int, w: int) -> int:
    return int(load().zvc_workspace_bytes(n, w))


def zvc_check_stream(h_comp: torch.Tensor, nbytes: int, n: int, w: int) -> int:
    """Host-side consistency check of a compressed stream in a CPU uint8 tensor.
    Returns the status code (ZVC_OK or an error), it does not raise."""
    assert h_comp.device.type == "cpu" and h_comp.is_contiguous()
    return int(load().zvc_check_stream(h_comp.data_ptr(), nbytes, n, w))


def zvc_window_check_stream(h_stream: torch.Tensor, nbytes: int, h_offsets: torch.Tensor, n: int,
                            w: int, window_bytes: int = WINDOW_PAPER_BYTES) -> int:
    """Host-side consistency check of a windowed stream (CPU uint8 tensor) and its table (CPU
    int64 tensor).  Returns the status code, it does not raise."""
    assert h_stream.device.type == "cpu" and h_offsets.device.type == "cpu"
    assert h_stream.is_contiguous() and h_offsets.is_contiguous() and h_offsets.dtype == torch.int64
    return int(load().zvc_window_check_stream(h_stream.data_ptr(), nbytes, h_offsets.data_ptr(), n, w,
                                              window_bytes))


def zvc_workspace_set_lookback_patience(ws: torch.Tensor, polls: int, stream=None) -> None:
    _check(load().zvc_workspace_set_lookback_patience(ws.data_ptr(), int(polls), _stream_handle(stream)),
           "zvc_workspace_set_lookback_patience")


def zvc_reference_stream(src: torch.Tensor, read_bytes: int, dst: torch.Tensor, write_bytes: int,
                         stream=None) -> None:
    """Enqueue the plain streaming kernel (measurement aid): read_bytes from src, write_bytes to dst."""
    _check(load().zvc_reference_stream(src.data_ptr(), read_bytes, dst.data_ptr(), write_bytes,
                                       _stream_handle(stream)), "zvc_reference_stream")


def zvc_workspace_self_help_count(ws: torch.Tensor) -> int:
    count = ctypes.c_uint64(0)
    _check(load().zvc_workspace_self_help_count(ws.data_ptr(), ctypes.byref(count)),
           "zvc_workspace_self_help_count")
    return int(count.value)


# ---- buffers -------------------------------------------------------------------
def new_workspace(n: int, w: int, device="cuda", stream=None) -> torch.Tensor:
    """Allocate and initialise a workspace big enough for n elements of width w."""
    nbytes = max(zvc_workspace_bytes(n, w), zvc_workspace_bytes(0, 4))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    zvc_workspace_init(ws, stream)
    return ws


def new_compressed_buffer(n: int, w: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(zvc_max_compressed_bytes(n, w), 16), dtype=torch.uint8, device=device)


# ---- device entry points ----------------------------------------------------------
def zvc_workspace_init(ws: torch.Tensor, stream=None) -> None:
    _check(load().zvc_workspace_init(ws.data_ptr(), ws.numel() * ws.element_size(),
                                     _stream_handle(stream)), "zvc_workspace_init")


def zvc_compressed_size(x: torch.Tensor, d_bytes: torch.Tensor, ws: torch.Tensor,
                        stream=None, n: Optional[int] = None) -> None:
    """Enqueue the count-only pass; d_bytes (int64[1] on the device) receives the size."""
    n = x.numel() if n is None else n
    _check(load().zvc_compressed_size(x.data_ptr(), n, x.element_size(), d_bytes.data_ptr(),
                                      ws.data_ptr(), ws.numel(), _stream_handle(stream)),
           "zvc_compressed_size")


def zvc_compress(x: torch.Tensor, out: torch.Tensor, d_bytes: torch.Tensor, ws: torch.Tensor,
                 stream=None, n: Optional[int] = None) -> None:
    """Enqueue compression of x (any w-byte dtype, contiguous) into the uint8 buffer `out`."""
    n = x.numel() if n is None else n
    _check(load().zvc_compress(x.data_ptr(), n, x.element_size(), out.data_ptr(), out.numel(),
                               d_bytes.data_ptr(), ws.data_ptr(), ws.numel(),
                               _stream_handle(stream)), "zvc_compress")


STATIC_MAX_BYTES = 1 << 30   # ZVC_STATIC_MAX_BYTES of include/zvc.h


def zvc_compress_static(x: torch.Tensor, out: torch.Tensor, d_bytes: torch.Tensor, stream=None,
                        n: Optional[int] = None) -> None:
    """zvc_compress without a workspace argument: the scan state lives in an array inside the
    library (for callers that cannot allocate).  Calls on one GPU must not overlap."""
    n = x.numel() if n is None else n
    _check(load().zvc_compress_static(x.data_ptr(), n, x.element_size(), out.data_ptr(), out.numel(),
                                      d_bytes.data_ptr(), _stream_handle(stream)), "zvc_compress_static")


def zvc_relu_compress(x: torch.Tensor, out: torch.Tensor, d_bytes: torch.Tensor, ws: torch.Tensor,
                      stream=None, n: Optional[int] = None) -> None:
    """Enqueue compression of ReLU(x) (x: fp32, fp16 or bf16 pre-activations) into `out`."""
    n = x.numel() if n is None else n
    _check(load().zvc_relu_compress(x.data_ptr(), n, x.element_size(), out.data_ptr(), out.numel(),
                                    d_bytes.data_ptr(), ws.data_ptr(), ws.numel(),
                                    _stream_handle(stream)), "zvc_relu_compress")


def zvc_compress_bounded(x: torch.Tensor, out: torch.Tensor, d_bytes: torch.Tensor, ws: torch.Tensor,
                         relu: bool = False, stream=None, n: Optional[int] = None,
                         out_cap: Optional[int] = None) -> None:
    """Enqueue compression of x (relu: of ReLU(x)) into `out`, which may be smaller than the
    worst case; d_bytes receives the size needed, to be compared with the capacity."""
    n = x.numel() if n is None else n
    _check(load().zvc_compress_bounded(x.data_ptr(), n, x.element_size(), int(bool(relu)),
                                       out.data_ptr(), out.numel() if out_cap is None else out_cap,
                                       d_bytes.data_ptr(), ws.data_ptr(), ws.numel(),
                                       _stream_handle(stream)), "zvc_compress_bounded")


def zvc_window_count(n: int, w: int, window_bytes: int = WINDOW_PAPER_BYTES) -> int:
    return int(load().zvc_window_count(n, w, window_bytes))


def zvc_window_elements(w: int, window_bytes: int = WINDOW_PAPER_BYTES) -> int:
    """Elements per window; 0 for a width or window size the library does not take."""
    return int(load().zvc_window_elements(w, window_bytes))


def zvc_window_compress(x: torch.Tensor, out: torch.Tensor, offsets: torch.Tensor,
                        d_bytes: torch.Tensor, ws: torch.Tensor, stream=None,
                        window_bytes: int = WINDOW_PAPER_BYTES) -> None:
    """Enqueue compression of x into the paper-order windowed stream `out` (uint8) and its
    offset table `offsets` (int64, zvc_window_count + 1 entries)."""
    n = x.numel()
    if zvc_window_elements(x.element_size(), window_bytes) != 0 and \
            offsets.numel() < zvc_window_count(n, x.element_size(), window_bytes) + 1:
        raise ZvcError(ZVC_E_CAPACITY, "zvc_window_compress (offset table too small)")
    _check(load().zvc_window_compress(x.data_ptr(), n, x.element_size(), window_bytes, out.data_ptr(),
                                      out.numel(), offsets.data_ptr(), d_bytes.data_ptr(), ws.data_ptr(),
                                      ws.numel(), _stream_handle(stream)), "zvc_window_compress")


def zvc_window_decompress(comp: torch.Tensor, comp_bytes: int, offsets: torch.Tensor, n: int,
                          first_window: int, num_windows: int, out: torch.Tensor, stream=None,
                          window_bytes: int = WINDOW_PAPER_BYTES) -> None:
    """Enqueue decompression of a range of windows into `out` (the elements of those windows)."""
    w = out.element_size()
    per = zvc_window_elements(w, window_bytes)
    need = max(0, min(n, (first_window + num_windows) * per) - first_window * per)
    if out.numel() < need:
        raise ZvcError(ZVC_E_CAPACITY, "zvc_window_decompress (output holds %d elements, %d needed)"
                       % (out.numel(), need))
    _check(load().zvc_window_decompress(comp.data_ptr(), comp_bytes, offsets.data_ptr(), n, w, window_bytes,
                                        first_window, num_windows, out.data_ptr(),
                                        _stream_handle(stream)), "zvc_window_decompress")


def zvc_decompress(comp: torch.Tensor, comp_bytes: int, out: torch.Tensor, ws: torch.Tensor,
                   stream=None, n: Optional[int] = None) -> None:
    """Enqueue decompression of the first comp_bytes bytes of `comp` into `out`."""
    n = out.numel() if n is None else n
    _check(load().zvc_decompress(comp.data_ptr(), comp_bytes, n, out.element_size(),
                                 out.data_ptr(), ws.data_ptr(), ws.numel(),
                                 _stream_handle(stream)), "zvc_decompress")


def zvc_offload(x: torch.Tensor, stage: torch.Tensor, h_pinned: torch.Tensor,
                h_bytes: torch.Tensor, ws: torch.Tensor, compute: torch.cuda.Stream,
                copy: torch.cuda.Stream) -> int:
    """Compress x into `stage` on `compute`, then copy exactly the compressed bytes to the
    pinned host tensor on `copy`.  Returns the compressed size (the call waits for it)."""
    _check(load().zvc_offload(x.data_ptr(), x.numel(), x.element_size(), stage.data_ptr(),
                              stage.numel(), h_pinned.data_ptr(), h_pinned.numel(),
                              h_bytes.data_ptr(), ws.data_ptr(), ws.numel(),
                              _stream_handle(compute), _stream_handle(copy)), "zvc_offload")
    return int(h_bytes.item())


def zvc_relu_offload(x: torch.Tensor, stage: torch.Tensor, h_pinned: torch.Tensor,
                     h_bytes: torch.Tensor, ws: torch.Tensor, compute: torch.cuda.Stream,
                     copy: torch.cuda.Stream) -> int:
    """zvc_offload with the fused ReLU encoder: x holds pre-activations, the host gets the
    stream of ReLU(x)."""
    _check(load().zvc_relu_offload(x.data_ptr(), x.numel(), x.element_size(), stage.data_ptr(),
                                   stage.numel(), h_pinned.data_ptr(), h_pinned.numel(),
                                   h_bytes.data_ptr(), ws.data_ptr(), ws.numel(),
                                   _stream_handle(compute), _stream_handle(copy)), "zvc_relu_offload")
    return int(h_bytes.item())


def zvc_prefetch(h_pinned: torch.Tensor, nbytes: int, stage: torch.Tensor, out: torch.Tensor,
                 ws: torch.Tensor, copy: torch.cuda.Stream, compute: torch.cuda.Stream) -> None:
    """Copy nbytes of compressed data back to `stage` on `copy`, then decompress into `out`
    on `compute` (ordered after the copy)."""
    _check(load().zvc_prefetch(h_pinned.data_ptr(), nbytes, out.numel(), out.element_size(),
                               stage.data_ptr(), stage.numel(), out.data_ptr(), ws.data_ptr(),
                               ws.numel(), _stream_handle(copy), _stream_handle(compute)),
           "zvc_prefetch")


def compress_tensor(x: torch.Tensor, ws: Optional[torch.Tensor] = None
                    ) -> Tuple[torch.Tensor, int]:
    """Convenience for tests: compress x, wait, return (buffer, compressed_bytes)."""
    n, w = x.numel(), x.element_size()
    ws = ws if ws is not None else new_workspace(n, w, x.device)
    out = new_compressed_buffer(n, w, x.device)
    d_bytes = torch.zeros(1, dtype=torch.int64, device=x.device)
    zvc_compress(x, out, d_bytes, ws)
    return out, int(d_bytes.item())
