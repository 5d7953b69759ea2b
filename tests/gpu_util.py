"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI
binding and compare with the CPU oracle, bit for bit."""
import sys

import numpy as np
import torch

from paper_1705_01626_amd import zvc


def say(msg):
    """Name the case before the GPU step runs, so a fault can be traced."""
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


def raw_bytes(t: torch.Tensor) -> np.ndarray:
    """The tensor's memory image as a numpy uint8 array (host copy)."""
    return t.contiguous().view(torch.uint8).cpu().numpy().reshape(-1)


def gpu_round_trip(x: torch.Tensor, ws=None, check_size_pass=True):
    """Compress + decompress x on the GPU.  Returns dict of host results."""
    n, w = x.numel(), x.element_size()
    dev = x.device
    ws = ws if ws is not None else zvc.new_workspace(n, w, dev)
    comp = zvc.new_compressed_buffer(n, w, dev)
    comp.fill_(0xCD)
    d_bytes = torch.full((1,), -1, dtype=torch.int64, device=dev)
    zvc.zvc_compress(x, comp, d_bytes, ws)
    nbytes = int(d_bytes.item())
    res = {"bytes": nbytes, "comp": comp, "ws": ws}
    if check_size_pass:
        d2 = torch.full((1,), -1, dtype=torch.int64, device=dev)
        zvc.zvc_compressed_size(x, d2, ws)
        res["size_pass"] = int(d2.item())
    out = torch.empty_like(x)
    out.view(torch.uint8).fill_(0xEE)
    zvc.zvc_decompress(comp, nbytes, out, ws)
    torch.cuda.synchronize()
    res["stream"] = comp[:nbytes].cpu().numpy()
    res["out"] = out
    return res


def assert_parity(x: torch.Tensor, oracle, label: str, ws=None):
    """Zero-tolerance comparison of masks, packed values, size and reconstruction."""
    n, w = x.numel(), x.element_size()
    say("%s n=%d w=%d ptr%%16=%d" % (label, n, w, x.data_ptr() % 16))
    host = raw_bytes(x)
    expect = oracle.compress_stream(host, w)
    res = gpu_round_trip(x, ws)
    G = (n + 31) // 32
    assert res["bytes"] == expect.size, "%s: size %d != oracle %d" % (label, res["bytes"], expect.size)
    assert res["size_pass"] == expect.size, "%s: count-only size" % label
    got = res["stream"]
    assert np.array_equal(got[: 4 * G], expect[: 4 * G]), "%s: mask words differ" % label
    assert np.array_equal(got[4 * G:], expect[4 * G:]), "%s: packed values differ" % label
    back = raw_bytes(res["out"])
    assert np.array_equal(back, host), "%s: reconstructed tensor differs" % label
    # and the oracle's decoder agrees with the GPU encoder's stream
    assert np.array_equal(oracle.decompress_stream(got, n, w), host)
    return res
