"""GPU parity of the fused ReLU + ZVC entry point against the CPU oracle
(ZVC stream of ReLU(x)), bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_1705_01626_amd import workloads, zvc
from tests.gpu_util import raw_bytes, say

pytestmark = pytest.mark.gpu
DEV = "cuda"
DTYPES = {4: torch.int32, 2: torch.int16}
SIZES = [0, 1, 31, 32, 33, 255, 4096, 4097, 8193, 100003, (1 << 20) + 5, 5 * (1 << 20) + 777, (1 << 24) + 8192 + 77]


def signed_words(n, w, zero_fraction, seed):
    """Random w-byte words of either sign (NaN, inf and denormal patterns included), some zeros."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    lo, hi = -(2 ** (8 * w - 1)), 2 ** (8 * w - 1)
    x = torch.randint(lo, hi, (n,), generator=g, dtype=torch.int64)
    x[torch.rand((n,), generator=g) < zero_fraction] = 0
    negzero = torch.rand((n,), generator=g) < 0.02
    x[negzero] = lo                                        # the pattern of -0.0
    return x.to(DTYPES[w]).to(DEV)


def relu_round_trip(x, ws=None):
    n, w = x.numel(), x.element_size()
    ws = ws if ws is not None else zvc.new_workspace(n, w, DEV)
    comp = zvc.new_compressed_buffer(n, w, DEV)
    comp.fill_(0xCD)
    d_bytes = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    zvc.zvc_relu_compress(x, comp, d_bytes, ws)
    nbytes = int(d_bytes.item())
    out = torch.empty_like(x)
    out.view(torch.uint8).fill_(0xEE)
    zvc.zvc_decompress(comp, nbytes, out, ws)
    torch.cuda.synchronize()
    return nbytes, comp[:nbytes].cpu().numpy(), out


def assert_relu_parity(x, oracle, label, ws=None):
    n, w = x.numel(), x.element_size()
    say("%s n=%d w=%d ptr%%16=%d" % (label, n, w, x.data_ptr() % 16))
    host = raw_bytes(x)
    expect = oracle.relu_compress_stream(host, w)
    nbytes, stream, out = relu_round_trip(x, ws)
    G = (n + 31) // 32
    assert nbytes == expect.size, "%s: size %d != oracle %d" % (label, nbytes, expect.size)
    assert np.array_equal(stream[: 4 * G], expect[: 4 * G]), "%s: mask words differ" % label
    assert np.array_equal(stream[4 * G:], expect[4 * G:]), "%s: packed values differ" % label
    assert np.array_equal(raw_bytes(out), oracle.relu(host, w)), "%s: decoded tensor is not ReLU(x)" % label
    return nbytes


@pytest.mark.parametrize("w", [4, 2])
@pytest.mark.parametrize("n", SIZES)
def test_relu_sizes(oracle, n, w):
    ws = zvc.new_workspace(max(n, 1), w, DEV)
    for k, zf in enumerate((0.0, 0.3, 0.9)):
        assert_relu_parity(signed_words(n, w, zf, seed=31 * n + k), oracle, "relu zf=%.1f" % zf, ws)


@pytest.mark.parametrize("w", [4, 2])
def test_relu_unaligned_pointer(oracle, w):
    for off, n in ((1, 37), (3, 20011), (5, 4096)):
        base = signed_words(n + 16, w, 0.3, seed=off * n)
        assert_relu_parity(base[off: off + n], oracle, "relu unaligned off=%d" % off)


def test_relu_special_values(oracle):
    """Signs of zero, infinities, NaNs of both signs, denormals (the reading of which patterns are positive)."""
    specials32 = [0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x7FC00000, 0xFFC00000, 0x7F800001,
                  0xFF800001, 0x00000001, 0x80000001, 0x007FFFFF, 0x807FFFFF, 0x3F800000, 0xBF800000]
    x = torch.from_numpy(np.array(specials32 * 700, dtype=np.uint32).view(np.int32)).to(DEV)
    assert_relu_parity(x, oracle, "relu specials fp32")
    specials16 = [0x0000, 0x8000, 0x7C00, 0xFC00, 0x7E00, 0xFE00, 0x0001, 0x8001, 0x3C00, 0xBC00, 0x7F80, 0xFF80]
    y = torch.from_numpy(np.array(specials16 * 900, dtype=np.uint16).view(np.int16)).to(DEV)
    assert_relu_parity(y, oracle, "relu specials 16-bit")


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16])
def test_relu_stream_equals_stream_of_relu_output(oracle, dtype):
    """Pre-activations of a blurred-field tensor: the fused call writes the very
    bytes zvc_compress writes for the ReLU output, and torch.relu agrees."""
    post = workloads.conv_small(seed=3, device=DEV)
    pre = workloads.pre_activation(post, seed=4).to(dtype)
    post_t = torch.relu(pre)
    n, w = pre.numel(), pre.element_size()
    ws = zvc.new_workspace(n, w, DEV)
    nbytes = assert_relu_parity(pre, oracle, "relu conv_small %s" % dtype, ws)
    comp = zvc.new_compressed_buffer(n, w, DEV)
    d_bytes = torch.zeros(1, dtype=torch.int64, device=DEV)
    zvc.zvc_compress(post_t, comp, d_bytes, ws)
    assert int(d_bytes.item()) == nbytes
    comp2 = zvc.new_compressed_buffer(n, w, DEV)
    zvc.zvc_relu_compress(pre, comp2, d_bytes, ws)
    torch.cuda.synchronize()
    assert torch.equal(comp[:nbytes], comp2[:nbytes])


def test_relu_conv1_style_full(oracle):
    """Full size of the benchmark tensor (297 MB, 64 KB tiles), element by element against the oracle."""
    post = workloads.conv1_style(seed=0, device=DEV)
    pre = workloads.pre_activation(post, seed=1)
    del post
    nbytes = assert_relu_parity(pre, oracle, "relu conv1_style full")
    n = pre.numel()
    d = (nbytes - n // 8) / 4 / n
    assert 0.45 < d < 0.56


def test_relu_offload_and_prefetch(oracle):
    """Pre-activations leave the GPU as the stream of their ReLU and come back as ReLU(x)."""
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    for dtype in (torch.float32, torch.bfloat16):
        post = workloads.conv_small(seed=6, device=DEV)
        pre = workloads.pre_activation(post, seed=7).to(dtype)
        n, w = pre.numel(), pre.element_size()
        cap = zvc.zvc_max_compressed_bytes(n, w)
        stage = torch.empty(cap, dtype=torch.uint8, device=DEV)
        h_pinned = torch.empty(cap, dtype=torch.uint8, pin_memory=True)
        h_bytes = torch.zeros(1, dtype=torch.int64, pin_memory=True)
        ws = zvc.new_workspace(n, w, DEV)
        torch.cuda.synchronize()
        say("relu offload %s" % dtype)
        nbytes = zvc.zvc_relu_offload(pre, stage, h_pinned, h_bytes, ws, compute, copy)
        copy.synchronize()
        expect = oracle.relu_compress_stream(raw_bytes(pre), w)
        assert nbytes == expect.size
        assert np.array_equal(h_pinned[:nbytes].numpy(), expect)
        stage.zero_()
        out = torch.empty_like(pre)
        torch.cuda.synchronize()
        zvc.zvc_prefetch(h_pinned, nbytes, stage, out, ws, copy, compute)
        compute.synchronize()
        assert np.array_equal(raw_bytes(out), oracle.relu(raw_bytes(pre), w))
