"""GPU parity of the paper-order windowed stream (zvc_window_compress /
zvc_window_decompress) against the CPU oracle, bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_1705_01626_amd import workloads, zvc
from tests.gpu_util import raw_bytes, say
from tests.test_gpu_parity import random_tensor

pytestmark = pytest.mark.gpu
DEV = "cuda"
SIZES = [0, 1, 31, 32, 33, 1023, 1024, 1025, 2047, 2048, 2049, 4096 * 3 + 17, 100003, (1 << 20) + 5,
         5 * (1 << 20) + 777, (1 << 24) + 8192 + 77]
# section 6's window is 4 KB; section 7.1 goes up to 64 KB; 1 KB is the kernels' own unit
WINDOWS = [1024, 2048, 4096, 8192, 16384, 32768, 65536]
PAPER = zvc.WINDOW_PAPER_BYTES


def window_compress(x, ws=None, window=PAPER):
    n, w = x.numel(), x.element_size()
    ws = ws if ws is not None else zvc.new_workspace(max(n, 1), w, DEV)
    comp = zvc.new_compressed_buffer(n, w, DEV)
    comp.fill_(0xCD)
    K = zvc.zvc_window_count(n, w, window)
    offsets = torch.full((K + 1,), -1, dtype=torch.int64, device=DEV)
    d_bytes = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    zvc.zvc_window_compress(x, comp, offsets, d_bytes, ws, window_bytes=window)
    torch.cuda.synchronize()
    return comp, offsets, int(d_bytes.item())


def some_ranges(K):
    return [(0, 1), (K - 1, 1), (K // 2, min(3, K - K // 2)), (K, 0)] if K > 0 else [(0, 0)]


def assert_window_parity(x, oracle, label, ws=None, ranges=None, window=PAPER):
    n, w = x.numel(), x.element_size()
    say("%s n=%d w=%d window=%d ptr%%16=%d" % (label, n, w, window, x.data_ptr() % 16))
    host = raw_bytes(x)
    per = zvc.zvc_window_elements(w, window)
    assert per * w == window
    expect, expect_offsets = oracle.window_compress(host, w, per)
    comp, offsets, nbytes = window_compress(x, ws, window)
    K = zvc.zvc_window_count(n, w, window)
    ranges = some_ranges(K) if ranges is None else ranges
    assert K == oracle.window_count(n, per)
    assert nbytes == expect.size, "%s: size %d != oracle %d" % (label, nbytes, expect.size)
    assert offsets.cpu().numpy().astype(np.uint64).tolist() == expect_offsets.tolist(), "%s: offset table" % label
    assert np.array_equal(comp[:nbytes].cpu().numpy(), expect), "%s: stream bytes differ" % label
    # whole tensor back
    out = torch.empty_like(x)
    out.view(torch.uint8).fill_(0xEE)
    zvc.zvc_window_decompress(comp, nbytes, offsets, n, 0, K, out, window_bytes=window)
    torch.cuda.synchronize()
    assert np.array_equal(raw_bytes(out), host), "%s: reconstructed tensor differs" % label
    # ranges of windows, each into a buffer of its own size
    for first, count in ranges:
        lo, hi = first * per, min(n, (first + count) * per)
        part = torch.empty(max(hi - lo, 0), dtype=x.dtype, device=DEV)
        part.view(torch.uint8).fill_(0x77)
        zvc.zvc_window_decompress(comp, nbytes, offsets, n, first, count, part, window_bytes=window)
        torch.cuda.synchronize()
        assert np.array_equal(raw_bytes(part), host[lo * w: hi * w]), "%s: windows %d+%d" % (label, first, count)
        assert np.array_equal(raw_bytes(part), oracle.window_decompress(expect, expect_offsets, n, w, per, first, count))
    return comp, offsets, nbytes


@pytest.mark.parametrize("w", [4, 2])
@pytest.mark.parametrize("n", SIZES)
def test_window_sizes_and_densities(oracle, n, w):
    """The paper's 4 KB window at every size and density; the kernels' 1 KB unit and a large
    window (a wave walks several 4 KB pieces) on the mixed density."""
    ws = zvc.new_workspace(max(n, 1), w, DEV)
    for k, density in enumerate((0.0, 0.35, 1.0)):
        x = random_tensor(n, w, density, seed=n * 7 + k)
        assert_window_parity(x, oracle, "window d=%.2f" % density, ws)
        if k == 1:
            assert_window_parity(x, oracle, "window d=%.2f" % density, ws, window=1024)
            assert_window_parity(x, oracle, "window d=%.2f" % density, ws, window=16384)


@pytest.mark.parametrize("w", [4, 2])
@pytest.mark.parametrize("window", WINDOWS)
def test_every_window_size(oracle, window, w):
    """All seven window sizes: a tensor of several windows with a ragged last one (ragged within
    a 1 KB unit, within a 4 KB piece and within the window), a tensor shorter than one window,
    and one that ends exactly on a window."""
    per = window // w
    for n in (5 * per + 3 * (1024 // w) + 77, per // 2 + 5, 3 * per, (1 << 21) + 4096 // w + 9):
        ws = zvc.new_workspace(n, w, DEV)
        for k, density in enumerate((0.35, 1.0, 0.02)):
            x = random_tensor(n, w, density, seed=window + n + k)
            assert_window_parity(x, oracle, "every window d=%.2f" % density, ws, window=window)


def test_table_of_a_larger_window_is_a_stride_of_a_smaller_ones(oracle):
    """The stream's bytes do not depend on the window size, and the 4 KB table is every fourth
    entry of the 1 KB table plus the total (oracle and kernel alike)."""
    n, w = 300007, 4
    x = random_tensor(n, w, 0.4, seed=77)
    comp1, off1, bytes1 = window_compress(x, window=1024)
    comp4, off4, bytes4 = window_compress(x, window=4096)
    assert bytes1 == bytes4 and torch.equal(comp1[:bytes1], comp4[:bytes4])
    assert off4[:-1].tolist() == off1[:-1:4].tolist() and int(off4[-1]) == int(off1[-1]) == bytes1
    host = raw_bytes(x)
    e1, o1 = oracle.window_compress(host, w, 1024 // w)
    e4, o4 = oracle.window_compress(host, w, 4096 // w)
    assert np.array_equal(e1, e4) and o4[:-1].tolist() == o1[:-1:4].tolist()


@pytest.mark.parametrize("w", [4, 2])
def test_window_unaligned_pointers(oracle, w):
    for off, n in ((1, 37), (3, 20011), (5, 4096)):
        base = random_tensor(n + 16, w, 0.35, seed=n + off)
        for window in (1024, PAPER, 65536):
            assert_window_parity(base[off: off + n], oracle, "window unaligned off=%d" % off, ranges=[(0, 1)],
                                 window=window)


def test_window_stream_has_the_planar_bytes_count(oracle):
    """Same size as the planar stream; masks and values inside are the planar ones (checked by the oracle's pins)."""
    x = workloads.conv_small(seed=5, device=DEV)
    n, w = x.numel(), 4
    ws = zvc.new_workspace(n, w, DEV)
    _, _, nbytes = assert_window_parity(x, oracle, "window conv_small", ws, [(3, 5)])
    comp = zvc.new_compressed_buffer(n, w, DEV)
    d_bytes = torch.zeros(1, dtype=torch.int64, device=DEV)
    zvc.zvc_compress(x, comp, d_bytes, ws)
    assert int(d_bytes.item()) == nbytes


@pytest.mark.parametrize("window", [1024, 2048, PAPER, 16384])
def test_window_decoder_stays_in_bounds_on_damaged_table(oracle, window):
    """A table that points past the stream, or claims oversized windows, must not make the
    kernel read outside the stream: it decodes what is there (zeros beyond)."""
    n, w = 200000, 4
    x = random_tensor(n, w, 0.5, seed=99)
    comp, offsets, nbytes = window_compress(x, window=window)
    K = zvc.zvc_window_count(n, w, window)
    bad = offsets.clone()
    bad[K // 2:] = nbytes + (1 << 40)          # far past the end
    out = torch.empty_like(x)
    say("damaged table window=%d" % window)
    zvc.zvc_window_decompress(comp, nbytes, bad, n, 0, K, out, window_bytes=window)
    torch.cuda.synchronize()
    per = window // w
    good = (K // 2 - 1) * per                   # windows whose both table entries are intact
    assert torch.equal(out[:good], x[:good])
    # window K//2 - 1 has a wrong end: clamped to the stream, its own bytes still decode
    assert torch.equal(out[good: good + per], x[good: good + per])
    assert not out[(K // 2) * per:].any()


def test_window_argument_errors_before_any_launch():
    x = torch.zeros(5000, dtype=torch.float32, device=DEV)
    K = zvc.zvc_window_count(5000, 4)
    comp, offsets, nbytes = window_compress(x)
    out = torch.empty_like(x)
    with pytest.raises(zvc.ZvcError):
        zvc.zvc_window_decompress(comp, nbytes, offsets, 5000, K, 1, out)      # past the last window
    with pytest.raises(zvc.ZvcError):
        zvc.zvc_window_decompress(comp, nbytes, offsets, 5000, 0, K + 1, out)
    small = torch.zeros(K, dtype=torch.int64, device=DEV)
    with pytest.raises(zvc.ZvcError):
        zvc.zvc_window_compress(x, comp, small, torch.zeros(1, dtype=torch.int64, device=DEV), zvc.new_workspace(5000, 4, DEV))
    # window sizes the library does not take: not a power of two, below 1 KB, above 64 KB
    big = torch.zeros(64, dtype=torch.int64, device=DEV)
    for window in (0, 512, 3072, 4095, 131072):
        assert zvc.zvc_window_count(5000, 4, window) == 0 and zvc.zvc_window_elements(4, window) == 0
        with pytest.raises(zvc.ZvcError) as err:
            zvc.zvc_window_compress(x, comp, big, torch.zeros(1, dtype=torch.int64, device=DEV),
                                    zvc.new_workspace(5000, 4, DEV), window_bytes=window)
        assert err.value.status == zvc.ZVC_E_ARG
        with pytest.raises(zvc.ZvcError) as err:
            zvc.zvc_window_decompress(comp, nbytes, offsets, 5000, 0, 1, out, window_bytes=window)
        assert err.value.status == zvc.ZVC_E_ARG


def test_window_conv1_style_full(oracle):
    """Full size of the benchmark tensor (297 MB) at the paper's window (72,600 windows of 4 KB),
    at the kernels' unit and at the largest window."""
    x = workloads.conv1_style(seed=0, device=DEV)
    K = zvc.zvc_window_count(x.numel(), 4, PAPER)
    assert K == 72600
    assert_window_parity(x, oracle, "window conv1_style full", ranges=[(0, 1), (12345, 1000), (K - 2, 2)])
    K1 = zvc.zvc_window_count(x.numel(), 4, 1024)
    assert K1 == 290400
    assert_window_parity(x, oracle, "window conv1_style full", ranges=[(12345, 1000), (K1 - 2, 2)], window=1024)
    K64 = zvc.zvc_window_count(x.numel(), 4, 65536)
    assert_window_parity(x, oracle, "window conv1_style full", ranges=[(777, 100), (K64 - 2, 2)], window=65536)


@pytest.mark.parametrize("window", [1024, PAPER, 32768])
def test_window_decoder_survives_garbage_stream_and_table(window):
    """Random bytes as the stream (with a genuine table) and random numbers as the table (with a
    genuine stream): every read is clamped to the stream and to the staged bytes, so the kernel
    finishes normally whatever it decodes.  Then a genuine call must still work."""
    n, w = 300000, 4
    x = random_tensor(n, w, 0.5, seed=4)
    comp, offsets, nbytes = window_compress(x, window=window)
    K = zvc.zvc_window_count(n, w, window)
    g = torch.Generator(device="cpu").manual_seed(8)
    junk = torch.randint(0, 256, (comp.numel(),), generator=g, dtype=torch.uint8).to(DEV)
    out = torch.empty_like(x)
    say("garbage stream")
    zvc.zvc_window_decompress(junk, nbytes, offsets, n, 0, K, out, window_bytes=window)
    torch.cuda.synchronize()
    wild = torch.randint(0, 1 << 62, (K + 1,), generator=g, dtype=torch.int64).to(DEV)
    say("garbage table")
    zvc.zvc_window_decompress(comp, nbytes, wild, n, 0, K, out, window_bytes=window)
    torch.cuda.synchronize()
    wild_small = torch.randint(0, nbytes, (K + 1,), generator=g, dtype=torch.int64).to(DEV)
    say("garbage table inside the stream")
    zvc.zvc_window_decompress(comp, nbytes, wild_small, n, 0, K, out, window_bytes=window)
    torch.cuda.synchronize()
    zvc.zvc_window_decompress(comp, nbytes, offsets, n, 0, K, out, window_bytes=window)
    torch.cuda.synchronize()
    assert torch.equal(out, x)


@pytest.mark.parametrize("w", [4, 2])
def test_window_dense_large_ranges(oracle, w):
    """Dense streams of ranges of 64 MB and more take the decoder's interleaved order:
    whole tensor and a large range that starts in the middle, ragged end."""
    n = 36 * (1 << 20) + 12345
    ws = zvc.new_workspace(n, w, DEV)
    x = random_tensor(n, w, 0.92, seed=1234 + w)
    for window in (1024, PAPER, 8192):
        K = zvc.zvc_window_count(n, w, window)
        assert_window_parity(x, oracle, "dense large w=%d" % w, ws, [(3, K - 3), (K // 16, K - K // 16)],
                             window=window)
