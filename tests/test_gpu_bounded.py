"""GPU parity of zvc_compress_bounded (compression into a buffer below the worst
case, for streams that stay in GPU memory) against the CPU oracle, through the
C ABI.  Where the stream fits, the buffer must hold the oracle's stream bit for
bit; where it does not, the size must still be the oracle's, the masks must be
complete and nothing may be written at or past the capacity."""
import numpy as np
import pytest
import torch

from paper_1705_01626_amd import workloads, zvc
from tests.gpu_util import raw_bytes, say
from tests.test_gpu_relu import signed_words

pytestmark = pytest.mark.gpu
DEV = "cuda"
GUARD = 4096
SIZES = [1, 32, 33, 4097, 100003, (1 << 20) + 5, (1 << 24) + 8192 + 77, 7 * (1 << 22)]


def oracle_stream(oracle, host, w, relu):
    return oracle.relu_compress_stream(host, w) if relu else oracle.compress_stream(host, w)


def bounded_call(x, cap, relu, ws):
    """Runs the call on a buffer of `cap` bytes followed by a guard area; returns
    (size reported, the cap bytes, whether the guard is untouched)."""
    buf = torch.full((cap + GUARD,), 0xA7, dtype=torch.uint8, device=DEV)
    d_bytes = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    zvc.zvc_compress_bounded(x, buf, d_bytes, ws, relu=relu, out_cap=cap)
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    return int(d_bytes.item()), got[:cap], bool((got[cap:] == 0xA7).all())


@pytest.mark.parametrize("relu", [False, True], ids=["plain", "relu"])
@pytest.mark.parametrize("w", [4, 2])
def test_bounded_exact_fit_and_too_small(oracle, w, relu):
    for n in SIZES:
        for zero_fraction in ((0.95, 0.5, 0.0) if n < (1 << 24) else (0.6,)):
            x = signed_words(n, w, zero_fraction, seed=n + w)
            host = raw_bytes(x)
            expect = oracle_stream(oracle, host, w, relu)
            masks = zvc.zvc_mask_bytes(n)
            ws = zvc.new_workspace(n, w, DEV)
            say("bounded n=%d w=%d relu=%s zeros=%.2f need=%d" % (n, w, relu, zero_fraction, expect.size))
            # exactly the size of the stream
            size, got, guard_ok = bounded_call(x, expect.size, relu, ws)
            assert size == expect.size and guard_ok
            assert np.array_equal(got, expect)
            # decodes from the exact-fit buffer
            comp = torch.from_numpy(got.copy()).to(DEV)
            out = torch.empty_like(x)
            zvc.zvc_decompress(comp, size, out, ws)
            torch.cuda.synchronize()
            want = oracle.relu(host, w) if relu else host
            assert np.array_equal(raw_bytes(out), want)
            # too small by one element, by half, and masks only: size still right, masks
            # complete, nothing past the capacity
            values = expect.size - masks
            for cap in {expect.size - w, masks + (values // 2 // 4) * 4, masks}:
                if cap < masks or cap >= expect.size:
                    continue
                size, got, guard_ok = bounded_call(x, cap, relu, ws)
                assert size == expect.size, (n, cap)
                assert guard_ok, (n, cap)
                assert np.array_equal(got[:masks], expect[:masks])
            # the same workspace serves an unbounded call afterwards
            full = zvc.new_compressed_buffer(n, w, DEV)
            d_bytes = torch.zeros(1, dtype=torch.int64, device=DEV)
            (zvc.zvc_relu_compress if relu else zvc.zvc_compress)(x, full, d_bytes, ws)
            assert int(d_bytes.item()) == expect.size
            assert np.array_equal(full[:expect.size].cpu().numpy(), expect)


def test_bounded_two_pass_footprint(oracle):
    """Count first, allocate exactly, compress: the stream in GPU memory takes
    compressed_bytes instead of the tensor's size."""
    x = workloads.conv_small(seed=3, device=DEV, batch=4)
    n, w = x.numel(), x.element_size()
    ws = zvc.new_workspace(n, w, DEV)
    d_bytes = torch.zeros(1, dtype=torch.int64, device=DEV)
    zvc.zvc_compressed_size(x, d_bytes, ws)
    need = int(d_bytes.item())
    assert need < n * w
    comp = torch.empty(need, dtype=torch.uint8, device=DEV)
    zvc.zvc_compress_bounded(x, comp, d_bytes, ws)
    assert int(d_bytes.item()) == need
    assert np.array_equal(comp.cpu().numpy(), oracle.compress_stream(raw_bytes(x), w))
    out = torch.empty_like(x)
    zvc.zvc_decompress(comp, need, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, x)


def test_bounded_empty_and_capacity_error():
    ws = zvc.new_workspace(0, 4, DEV)
    d_bytes = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    x = torch.empty(0, dtype=torch.float32, device=DEV)
    zvc.zvc_compress_bounded(x, torch.empty(16, dtype=torch.uint8, device=DEV), d_bytes, ws)
    assert int(d_bytes.item()) == 0
    x = torch.ones(1000, dtype=torch.float32, device=DEV)
    ws = zvc.new_workspace(1000, 4, DEV)
    with pytest.raises(zvc.ZvcError) as err:
        zvc.zvc_compress_bounded(x, torch.empty(zvc.zvc_mask_bytes(1000) - 4, dtype=torch.uint8, device=DEV),
                                 d_bytes, ws)
    assert err.value.status == zvc.ZVC_E_CAPACITY
