"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.
Bit-exact on mask words, packed values, compressed size and reconstruction."""
import numpy as np
import pytest
import torch

from paper_1705_01626_amd import workloads, zvc
from tests.gpu_util import assert_parity, raw_bytes, say

pytestmark = pytest.mark.gpu

DEV = "cuda"
SIZES = [0, 1, 2, 31, 32, 33, 63, 64, 65, 255, 256, 257, 4095, 4096, 4097, 8191, 8192, 8193,
         3 * 4096 + 17, 5 * 8192 - 1, 100003, (1 << 20) + 5,
         5 * (1 << 20) + 777, (1 << 24) + 8192 + 77]  # the last two reach the 32 KB and 64 KB tile kernels at either width
DTYPES = {4: torch.int32, 2: torch.int16}


def random_tensor(n, w, density, seed, device=DEV):
    g = torch.Generator(device="cpu").manual_seed(seed)
    hi = 2 ** (8 * w - 1) - 1
    x = torch.randint(1, hi, (n,), generator=g, dtype=torch.int64)
    sign = torch.randint(0, 2, (n,), generator=g, dtype=torch.int64) * 2 - 1
    keep = torch.rand((n,), generator=g) < density
    x = (x * sign * keep).to(DTYPES[w])
    return x.to(device)


@pytest.mark.parametrize("w", [4, 2])
@pytest.mark.parametrize("n", SIZES)
def test_sizes_and_densities(oracle, n, w):
    ws = zvc.new_workspace(max(n, 1), w, DEV)
    for k, density in enumerate((0.0, 0.03, 0.4, 0.97, 1.0)):
        x = random_tensor(n, w, density, seed=n * 10 + k)
        assert_parity(x, oracle, "random d=%.2f" % density, ws)  # workspace reused across calls


@pytest.mark.parametrize("w", [4, 2])
@pytest.mark.parametrize("offset_elems", [1, 2, 3, 5])
def test_unaligned_tensor_pointers(oracle, w, offset_elems):
    """Input/output pointers aligned only to the element width."""
    for n in (1, 37, 4096, 20011):
        base = random_tensor(n + 16, w, 0.35, seed=n + offset_elems)
        x = base[offset_elems: offset_elems + n]
        assert x.data_ptr() % 16 != 0 or w * offset_elems % 16 == 0
        say("unaligned n=%d w=%d off=%d" % (n, w, offset_elems))
        host = raw_bytes(x)
        expect = oracle.compress_stream(host, w)
        ws = zvc.new_workspace(n, w, DEV)
        comp = zvc.new_compressed_buffer(n, w, DEV)
        d_bytes = torch.zeros(1, dtype=torch.int64, device=DEV)
        zvc.zvc_compress(x, comp, d_bytes, ws)
        nbytes = int(d_bytes.item())
        assert nbytes == expect.size
        assert np.array_equal(comp[:nbytes].cpu().numpy(), expect)
        out_base = torch.zeros(n + 16, dtype=DTYPES[w], device=DEV)
        out = out_base[offset_elems: offset_elems + n]
        zvc.zvc_decompress(comp, nbytes, out, ws)
        torch.cuda.synchronize()
        assert np.array_equal(raw_bytes(out), host)
        # neighbours of the output range untouched
        assert int(out_base[:offset_elems].abs().sum()) == 0
        assert int(out_base[offset_elems + n:].abs().sum()) == 0


@pytest.mark.parametrize("w,n", [(4, 26000003), (2, 52000007)])
def test_32_kb_tile_kernels(oracle, w, n):
    """104 MB tensors (the 32 KB tile kernels at either width; the 64 KB ones run in the full-size
    sweep tests); ragged size, two densities."""
    ws = zvc.new_workspace(n, w, DEV)
    for k, density in enumerate((0.08, 0.6)):
        x = random_tensor(n, w, density, seed=n + k)
        assert_parity(x, oracle, "32 KB tiles d=%.2f" % density, ws)
        del x


def test_compressed_buffer_at_4_byte_alignment(oracle):
    """The compressed buffer only needs 4-byte alignment."""
    n, w = 50000, 4
    x = random_tensor(n, w, 0.5, seed=5)
    expect = oracle.compress_stream(raw_bytes(x), w)
    ws = zvc.new_workspace(n, w, DEV)
    for off in (4, 8, 12):
        big = torch.zeros(zvc.zvc_max_compressed_bytes(n, w) + 32, dtype=torch.uint8, device=DEV)
        comp = big[off: off + zvc.zvc_max_compressed_bytes(n, w)]
        d_bytes = torch.zeros(1, dtype=torch.int64, device=DEV)
        say("comp buffer offset %d" % off)
        zvc.zvc_compress(x, comp, d_bytes, ws)
        nbytes = int(d_bytes.item())
        assert np.array_equal(comp[:nbytes].cpu().numpy(), expect)
        out = torch.empty_like(x)
        zvc.zvc_decompress(comp, nbytes, out, ws)
        torch.cuda.synchronize()
        assert torch.equal(out, x)
        assert int(big[:off].sum()) == 0  # nothing written in front of the buffer


def test_special_bit_patterns(oracle):
    pats32 = torch.tensor([0x80000000, 0x7FC00000, 0x7F800001, 0xFFC12345, 0x00000001,
                           0x807FFFFF, 0x7F800000, 0xFF800000, 0x00000000, 0x3F800000],
                          dtype=torch.int64)
    x = pats32.repeat(1000).to(torch.int32).view(torch.float32).to(DEV)  # wraps to bit patterns
    res = assert_parity(x, oracle, "special fp32 patterns")
    assert res["bytes"] == 4 * ((x.numel() + 31) // 32) + 4 * 9000
    pats16 = torch.tensor([0x8000, 0x7E00, 0x7C01, 0x0001, 0x83FF, 0x7C00, 0xFC00, 0x0000,
                           0x3C00, 0xFFFF], dtype=torch.int64)
    y = pats16.repeat(1000).to(torch.int16).view(torch.float16).to(DEV)
    assert_parity(y, oracle, "special fp16 patterns")
    z = pats16.repeat(1000).to(torch.int16).view(torch.bfloat16).to(DEV)
    assert_parity(z, oracle, "special bf16 patterns")


def test_extremes(oracle):
    for w in (4, 2):
        for n in (32 * 128 * 7, 70001):
            z = torch.zeros(n, dtype=DTYPES[w], device=DEV)
            r = assert_parity(z, oracle, "all zero")
            assert r["bytes"] == 4 * ((n + 31) // 32)
            d = torch.full((n,), 7, dtype=DTYPES[w], device=DEV)
            r = assert_parity(d, oracle, "all dense")
            assert r["bytes"] == 4 * ((n + 31) // 32) + w * n


def test_workload_conv_small_full_size(oracle):
    """BASELINE config 0 at its full size (1.6 M elements)."""
    x = workloads.conv_small(seed=0, device=DEV)
    r = assert_parity(x, oracle, "conv_small 8x64x56x56")
    density = (r["bytes"] - 4 * (x.numel() // 32)) / 4 / x.numel()
    assert abs(density - 0.4) < 0.01


def test_workload_shapes_reduced_batch(oracle):
    """The other workloads' recipes at a reduced batch (several tiles, ragged planes)."""
    x = workloads.conv1_style(seed=1, device=DEV, batch=3)
    assert_parity(x, oracle, "conv1_style batch 3")
    for d in workloads.DENSITY_SWEEP:
        x = workloads.density_sweep(d, seed=2, device=DEV, batch=1)[:, :8]
        x = x.contiguous()
        r = assert_parity(x, oracle, "density sweep d=%.2f" % d)
        if d == 1.0:
            assert r["bytes"] == zvc.zvc_max_compressed_bytes(x.numel(), 4)
    variants = workloads.layout_variants(seed=3, device=DEV, batch=4)
    sizes = {}
    for name, t in variants.items():
        sizes[name] = assert_parity(t, oracle, "layout " + name)["bytes"]
    assert sizes["fp32_nchw"] == sizes["fp32_nhwc"] == sizes["fp32_chwn"]


def test_repeated_calls_on_one_workspace(oracle):
    """Many back-to-back launches reusing one workspace and one stream."""
    n, w = 300000, 4
    ws = zvc.new_workspace(n, w, DEV)
    comp = zvc.new_compressed_buffer(n, w, DEV)
    d_bytes = torch.zeros(1, dtype=torch.int64, device=DEV)
    xs = [random_tensor(n - 1000 * k, w, 0.1 + 0.2 * k, seed=k) for k in range(4)]
    expects = [oracle.compress_stream(raw_bytes(x), w) for x in xs]
    say("repeated calls")
    for rep in range(25):
        k = rep % 4
        zvc.zvc_compress(xs[k], comp, d_bytes, ws, n=xs[k].numel())
        nbytes = int(d_bytes.item())
        assert nbytes == expects[k].size
        if rep % 6 == 0:
            assert np.array_equal(comp[:nbytes].cpu().numpy(), expects[k])
        out = torch.empty_like(xs[k])
        zvc.zvc_decompress(comp, nbytes, out, ws)
        assert torch.equal(out, xs[k])


def test_offload_prefetch_round_trip(oracle):
    """compress -> pinned host -> back -> decompress on two streams."""
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    for w, n in ((4, 500000), (2, 123457), (4, 0)):
        x = random_tensor(n, w, 0.3, seed=n + w)
        torch.cuda.synchronize()
        cap = max(zvc.zvc_max_compressed_bytes(n, w), 16)
        stage = torch.empty(cap, dtype=torch.uint8, device=DEV)
        h_pinned = torch.empty(cap, dtype=torch.uint8, pin_memory=True)
        h_bytes = torch.zeros(1, dtype=torch.int64, pin_memory=True)
        ws = zvc.new_workspace(max(n, 1), w, DEV)
        torch.cuda.synchronize()
        say("offload n=%d w=%d" % (n, w))
        nbytes = zvc.zvc_offload(x, stage, h_pinned, h_bytes, ws, compute, copy)
        copy.synchronize()
        expect = oracle.compress_stream(raw_bytes(x), w)
        assert nbytes == expect.size
        assert np.array_equal(h_pinned[:nbytes].numpy(), expect)
        assert zvc.zvc_check_stream(h_pinned, nbytes, n, w) == zvc.ZVC_OK
        stage.fill_(0)
        out = torch.empty_like(x)
        torch.cuda.synchronize()
        zvc.zvc_prefetch(h_pinned, nbytes, stage, out, ws, copy, compute)
        compute.synchronize()
        assert torch.equal(out, x)


def test_decompress_never_reads_past_comp_bytes(oracle):
    """Masks that ask for more values than the stream holds decode the missing
    elements as zero (and read nothing past comp_bytes)."""
    n, w = 10000, 4
    x = random_tensor(n, w, 1.0, seed=9)
    comp, nbytes = zvc.compress_tensor(x)
    G = (n + 31) // 32
    cut = 4 * G + 4 * 6000  # pretend only 6000 values are present
    out = torch.empty_like(x)
    ws = zvc.new_workspace(n, w, DEV)
    say("truncated stream")
    zvc.zvc_decompress(comp, cut, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out[:6000], x[:6000])
    assert int(out[6000:].abs().sum()) == 0


def test_scan_wait_that_helps_itself(oracle):
    """With zero patience every wait in the device-wide scan computes the
    missing predecessor's count itself.  Results must not change, and every
    kernel still exits normally.  The setting belongs to the workspace."""
    helped = 0
    for w, n in ((4, 3000001), (2, 5000003), (4, 6000001), (4, (1 << 24) + 12345), (4, 100 * (1 << 20) + 3)):   # all three tile sizes
        x = random_tensor(n, w, 0.45, seed=w + n)
        ws = zvc.new_workspace(n, w, DEV)
        zvc.zvc_workspace_set_lookback_patience(ws, 0)
        res = assert_parity(x, oracle, "zero-patience scan", ws)
        helped += zvc.zvc_workspace_self_help_count(res["ws"])
        # another workspace keeps the default
        assert_parity(x[: n // 3], oracle, "default patience beside it")
    say("self-help events: %d" % helped)
    assert helped > 0


def test_single_launch_decoder_scan_that_helps_itself(oracle):
    """Tensors below 16 MB decode in one launch whose workgroups find their offsets with the
    device-wide scan.  With zero patience on the decoder's workspace (the stream comes from a call
    on another one) every wait computes the missing workgroup's popcount itself; the output must
    not change, and the workspace must be clean for the next call."""
    for w, n in ((4, 3999999), (2, 8000001), (4, 4194303), (4, 4194304), (2, 33)):   # up to the 16 MB limit and just past it
        x = random_tensor(n, w, 0.37, seed=n)
        res = assert_parity(x, oracle, "decoder input")
        ws = zvc.new_workspace(n, w, DEV)
        zvc.zvc_workspace_set_lookback_patience(ws, 0)
        out = torch.empty_like(x)
        out.view(torch.uint8).fill_(0x5A)
        say("zero-patience decode n=%d w=%d" % (n, w))
        zvc.zvc_decompress(res["comp"], res["bytes"], out, ws)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.uint8), x.view(torch.uint8))
        helped = zvc.zvc_workspace_self_help_count(ws)
        say("self-help events while decoding: %d" % helped)
        if n * w < (16 << 20) and n > 100000:
            assert helped > 0
        assert_parity(x, oracle, "the same workspace afterwards", ws)


def test_self_help_is_rare_in_normal_runs(oracle):
    """Default patience: predecessors publish long before a waiting tile gives
    up.  How often a count is computed twice depends on dispatch order and on
    what else the GPU is doing, so this reports the number and only checks that
    the fallback is not the normal path."""
    n, w = (1 << 24) + 4096, 4
    x = random_tensor(n, w, 0.5, seed=77)
    ws = zvc.new_workspace(n, w, DEV)
    comp = zvc.new_compressed_buffer(n, w, DEV)
    d_bytes = torch.zeros(1, dtype=torch.int64, device=DEV)
    say("self-help counter, compress")
    zvc.zvc_compress(x, comp, d_bytes, ws)
    torch.cuda.synchronize()
    helped = zvc.zvc_workspace_self_help_count(ws)
    say("self-help events at default patience: %d" % helped)
    tiles = (n * w + (32 << 10) - 1) // (32 << 10)
    assert helped <= tiles // 100
    out = torch.empty_like(x)
    zvc.zvc_decompress(comp, int(d_bytes.item()), out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, x)


def test_small_decode_then_large_encode_on_one_workspace(oracle):
    """The decoder's scratch arrays must not land where a later, larger encoder
    call on the same workspace keeps its scan state."""
    big_n, small_n, w = 40 * (1 << 20) + 5, 300007, 4
    ws = zvc.new_workspace(big_n, w, DEV)
    small = random_tensor(small_n, w, 0.999, seed=5)      # dense: large decoder prefix words
    res = assert_parity(small, oracle, "small tensor on a large workspace", ws)
    big = random_tensor(big_n, w, 0.3, seed=6)
    assert_parity(big, oracle, "large tensor after it", ws)
    out = torch.empty_like(small)
    zvc.zvc_decompress(res["comp"], res["bytes"], out, ws)
    assert_parity(big, oracle, "large tensor again, after a small decode", ws)
    torch.cuda.synchronize()
    assert torch.equal(out, small)


def test_decoder_many_chunks_and_reuse(oracle):
    """The decoder's pre-pass: one workgroup per 4096 masks, the last one to
    finish prefixes the chunk totals and resets its counter.  Sizes from one
    chunk to several hundred, the same workspace reused back to back."""
    w = 4
    n_max = 4096 * 32 * 300 + 12345
    ws = zvc.new_workspace(n_max, w, DEV)
    # (tensors below 16 MB decode in one launch, without the pre-pass: the sizes from 33 chunks up take it)
    for n in (4096 * 32, 4096 * 32 + 1, 4096 * 32 * 2 - 1, n_max, 4096 * 32 * 7 + 31, 1000,
              4096 * 32 * 33 - 1, 4096 * 32 * 40 + 5, 4096 * 32 * 32, 4096 * 32 * 32 - 1):
        x = random_tensor(n, w, 0.41, seed=n)
        assert_parity(x, oracle, "pre-pass chunks n=%d" % n, ws=ws)


def test_decoder_survives_garbage_stream(oracle):
    """Random bytes as a compressed stream: masks then claim any number of stored elements, but
    reads are clamped to comp_bytes and a step never stages more than it has room for, so the
    kernels finish normally; the workspace stays usable."""
    for w, n in ((4, 700001), (2, 1300003), (4, 6000011), (2, 9000001)):     # one launch | pre-pass + expand
        g = torch.Generator(device="cpu").manual_seed(n)
        cap = zvc.zvc_max_compressed_bytes(n, w)
        junk = torch.randint(0, 256, (cap,), generator=g, dtype=torch.uint8).to(DEV)
        ws = zvc.new_workspace(n, w, DEV)
        out = torch.empty(n, dtype=DTYPES[w], device=DEV)
        for comp_bytes in (cap, 4 * ((n + 31) // 32), 4 * ((n + 31) // 32) + w * (n // 3)):
            say("garbage stream w=%d comp_bytes=%d" % (w, comp_bytes))
            zvc.zvc_decompress(junk, comp_bytes, out, ws)
            torch.cuda.synchronize()
        x = random_tensor(n, w, 0.4, seed=1)
        assert_parity(x, oracle, "after garbage", ws)


@pytest.mark.parametrize("read_bytes,write_bytes", [(16, 16), (16, 0), (0, 4096), (16384 + 16, 48), (5 << 20, (3 << 20) + 16),
                                                     ((40 << 20) + 1040, 13 << 20), (9 << 20, (33 << 20) + 16)])
def test_reference_stream_kernel_stays_inside_its_buffers(read_bytes, write_bytes):
    """The benchmark's yardstick kernel: it writes every 16-byte chunk of [0, write_bytes) and
    nothing outside (guard bytes on both sides keep their value), whatever the two sizes are,
    and leaves its input alone."""
    guard = 4096
    src = torch.randint(1, 255, (read_bytes + 16,), dtype=torch.uint8, device=DEV)
    keep = src.clone()
    dst = torch.full((guard + write_bytes + guard,), 0xA5, dtype=torch.uint8, device=DEV)
    say("reference stream read=%d write=%d" % (read_bytes, write_bytes))
    zvc.zvc_reference_stream(src, read_bytes, dst[guard:], write_bytes)
    torch.cuda.synchronize()
    assert torch.equal(src, keep)
    assert bool((dst[:guard] == 0xA5).all()) and bool((dst[guard + write_bytes:] == 0xA5).all())
    if write_bytes:
        # a chunk whose 16 bytes all still hold the fill value was not written (the kernel writes a mix
        # of its input and the workgroup's number: 16 bytes of 0xA5 would be a coincidence of 2^-128)
        chunks = dst[guard: guard + write_bytes].view(-1, 16)
        assert not bool((chunks == 0xA5).all(dim=1).any())
