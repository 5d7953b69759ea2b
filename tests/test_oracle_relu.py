"""Pins for the oracle's fused ReLU + ZVC functions.  No GPU needed.

Checked against things other than the oracle itself: hand-worked fixtures,
library ReLU routines (numpy.maximum on float32, torch.relu on fp16/bf16) on
NaN-free inputs, the sign-and-zero rule spelled out on every 16-bit pattern,
and the composition property that defines the fused operation.
"""
import numpy as np
import pytest
import torch

from tests.golden_cases import load_relu_cases
from tests.test_oracle import library_zvc


@pytest.mark.parametrize("case", load_relu_cases(), ids=lambda c: c["name"])
def test_relu_handbuilt_cases(oracle, case):
    w, n = case["w"], case["n"]
    dense = oracle.relu(case["in"], w)
    assert dense.tobytes() == case["relu"].tobytes()
    stream = oracle.relu_compress_stream(case["in"], w)
    assert stream.size == case["bytes"]
    assert stream.tobytes() == case["masks"].astype("<u4").tobytes() + case["values"].tobytes()
    # the ordinary decoder gives back ReLU(in)
    assert oracle.decompress_stream(stream, n, w).tobytes() == case["relu"].tobytes()


def test_relu_matches_numpy_maximum_fp32(oracle):
    """max(x, 0) from the library on finite values, infinities, denormals and both zeros."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal(5003).astype(np.float32)
    x[:8] = [0.0, -0.0, np.inf, -np.inf, 1e-45, -1e-45, 3.0e38, -3.0e38]
    expect = np.maximum(x, np.float32(0.0))
    expect[x == 0] = 0.0                      # numpy may return either zero for max(-0, +0)
    got = oracle.relu(x, 4).view(np.float32)
    assert got.tobytes() == expect.tobytes()


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_relu_matches_torch_relu_16bit(oracle, dtype):
    g = torch.Generator().manual_seed(11)
    x = torch.randn(4099, generator=g).to(dtype)
    x[:6] = torch.tensor([0.0, -0.0, float("inf"), float("-inf"), 6e-8, -6e-8]).to(dtype)
    expect = torch.relu(x)
    expect[x == 0] = 0.0
    raw = x.view(torch.int16).numpy().view(np.uint16)
    got = oracle.relu(raw, 2).view(np.uint16)
    assert got.tobytes() == expect.view(torch.int16).numpy().tobytes()


def test_relu_rule_on_every_16bit_pattern(oracle):
    """Kept unchanged iff the sign bit is clear and the pattern is not +0; else +0."""
    words = np.arange(65536, dtype=np.uint16)
    got = oracle.relu(words, 2).view(np.uint16)
    for v in (0x0000, 0x8000, 0xFFFF, 0x8001, 0xFC00, 0xFE00):     # zeros, negatives, -inf, -NaN
        assert got[v] == 0
    for v in (0x0001, 0x3C00, 0x7BFF, 0x7C00, 0x7E00, 0x7FFF):     # denormal .. +inf, +NaN
        assert got[v] == v
    assert int(np.count_nonzero(got)) == 0x7FFF
    assert np.array_equal(got[1:0x8000], words[1:0x8000])
    assert not got[0x8000:].any()


@pytest.mark.parametrize("w", [2, 4])
@pytest.mark.parametrize("n", [0, 1, 31, 32, 33, 95, 4097])
def test_fused_is_zvc_of_relu(oracle, n, w):
    """Definition of the fused operation, with the ZVC step taken from the
    library-routine implementation (numpy bit packing and boolean selection)."""
    rng = np.random.default_rng(50 * n + w)
    dtype = np.uint32 if w == 4 else np.uint16
    words = rng.integers(0, 2 ** (8 * w), size=n, dtype=np.uint64).astype(dtype)
    words[rng.random(n) < 0.2] = 0
    sign = dtype(1 << (8 * w - 1))
    activated = np.where((words & sign) == 0, words, dtype(0)).astype(dtype)
    masks, values = library_zvc(activated)
    stream = oracle.relu_compress_stream(words, w)
    assert stream.tobytes() == masks.astype("<u4").tobytes() + values.tobytes()
    assert stream.tobytes() == oracle.compress_stream(oracle.relu(words, w), w).tobytes()
    assert oracle.relu(oracle.relu(words, w), w).tobytes() == oracle.relu(words, w).tobytes()   # idempotent


def test_relu_on_post_relu_input_changes_nothing(oracle):
    """A tensor that is already a ReLU output compresses the same either way."""
    rng = np.random.default_rng(3)
    x = np.maximum(rng.standard_normal(3001).astype(np.float32), 0)
    assert oracle.relu_compress_stream(x, 4).tobytes() == oracle.compress_stream(x, 4).tobytes()


def test_relu_bad_width_rejected(oracle):
    with pytest.raises(ValueError):
        oracle.relu(np.zeros(4, dtype=np.uint8), 3)
    with pytest.raises(ValueError):
        oracle.relu_compress_stream(np.zeros(8, dtype=np.uint8), 8)
