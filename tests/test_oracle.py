"""Pins for the CPU oracle (oracle/zvc_ref.cpp).  No GPU needed.

The oracle is checked against things other than itself: hand-worked fixtures,
numbers the paper states, closed forms, a second implementation built from
library routines (numpy bit packing and boolean selection), brute force, and
the invariants of the scheme (lossless round trip, layout independence).
"""
import numpy as np
import pytest

from tests.golden_cases import load_handbuilt, load_paper_numbers

RAGGED_SIZES = [0, 1, 31, 32, 33, 63, 64, 65, 95, 96, 1000, 4095, 4096, 4097, 12345]


# --------------------------------------------------------------------------
# an independent second implementation made of library routines only
# --------------------------------------------------------------------------
def library_zvc(words: np.ndarray):
    """words: uint16/uint32 element bit patterns.  Returns (masks, values)."""
    nz = words != 0
    n = words.size
    pad = (-n) % 32
    bits = np.concatenate([nz, np.zeros(pad, dtype=bool)])
    masks = np.packbits(bits, bitorder="little").view("<u4") if bits.size else np.zeros(0, "<u4")
    return masks.astype(np.uint32), words[nz]


def random_words(rng, n, w, density):
    dtype = np.uint32 if w == 4 else np.uint16
    hi = 2 ** (8 * w)
    x = rng.integers(1, hi, size=n, dtype=np.uint64).astype(dtype)
    keep = rng.random(n) < density
    return np.where(keep, x, 0).astype(dtype)


# --------------------------------------------------------------------------
# hand-worked fixtures
# --------------------------------------------------------------------------
@pytest.mark.parametrize("case", load_handbuilt(), ids=lambda c: c["name"])
def test_handbuilt_cases(oracle, case):
    masks, values, nnz = oracle.compress(case["in"], case["w"])
    assert masks.tolist() == case["masks"].tolist()
    assert values.view(case["in"].dtype).tolist() == case["values"].tolist()
    assert nnz == case["values"].size
    assert oracle.compressed_bytes(case["n"], case["w"], nnz) == case["bytes"]
    stream = oracle.compress_stream(case["in"], case["w"])
    assert stream.size == case["bytes"]
    expect = case["masks"].astype("<u4").tobytes() + case["values"].tobytes()
    assert stream.tobytes() == expect
    back = oracle.decompress_stream(stream, case["n"], case["w"])
    assert back.tobytes() == case["in"].tobytes()


# --------------------------------------------------------------------------
# what the paper states (section 5.1, 5.2, 7.1)
# --------------------------------------------------------------------------
def test_paper_all_zero_group_is_32x(oracle):
    paper = load_paper_numbers()
    x = np.zeros(32, dtype=np.float32)
    stream = oracle.compress_stream(x, 4)
    assert stream.size == 4 and not stream.any()
    assert x.nbytes / stream.size == paper["ratio_all_zero_group"]
    # many groups: still exactly 32x
    x = np.zeros(32 * 1000, dtype=np.float32)
    assert x.nbytes / oracle.compress_stream(x, 4).size == paper["ratio_all_zero_group"]


def test_paper_dense_group_overhead(oracle):
    paper = load_paper_numbers()
    x = np.arange(1, 33, dtype=np.float32)
    masks, values, nnz = oracle.compress(x, 4)
    assert masks.tolist() == [0xFFFFFFFF] and nnz == 32
    assert values.tobytes() == x.tobytes()
    size = oracle.compressed_bytes(32, 4, nnz)
    overhead = 100.0 * (size - x.nbytes) / x.nbytes
    assert overhead == paper["overhead_dense_group_percent"]
    assert abs(overhead - 3.1) < 0.05  # the paper's rounded figure


def test_paper_headline_ratios_follow_the_size_formula(oracle):
    """ratio = n*w / (4*ceil(n/32) + w*nnz).  The paper's 13.8x maximum and 2.6x
    average must be reachable: build tensors with the matching non-zero count
    and check the oracle's size gives those ratios."""
    paper = load_paper_numbers()
    n = 32 * 100000
    for target in (paper["max_layer_ratio"], paper["average_ratio"]):
        d = (32.0 / target - 1.0) / 32.0
        nnz = int(round(d * n))
        x = np.zeros(n, dtype=np.float32)
        x[np.linspace(0, n - 1, nnz).astype(np.int64)] = 1.0
        nnz = int(np.count_nonzero(x))
        stream = oracle.compress_stream(x, 4)
        assert stream.size == 4 * (n // 32) + 4 * nnz
        assert abs(x.nbytes / stream.size - target) < 0.01
    # 13.8x <=> about 4 % density; 2.6x <=> about 35 % density, i.e. close to
    # the 62 % average sparsity the paper reports
    assert abs((32 / paper["max_layer_ratio"] - 1) / 32 - 0.0412) < 1e-3
    d_avg = (32 / paper["average_ratio"] - 1) / 32
    assert abs((1 - d_avg) * 100 - paper["average_sparsity_percent"]) < 4.0
    assert paper["max_layer_ratio"] * 16 == pytest.approx(paper["crossbar_bandwidth_GBps"])


def test_paper_60_percent_zero_example(oracle):
    """40 % dense: values alone shrink 2.5x (the paper's figure, masks left
    out); with the masks the stream ratio is 32/(1+32*0.4)."""
    paper = load_paper_numbers()
    n = 32 * 5000
    x = np.zeros(n, dtype=np.float32)
    x[np.arange(n) % 5 < 2] = 7.0  # exactly 40 % non-zero
    masks, values, nnz = oracle.compress(x, 4)
    assert x.nbytes / values.size == paper["ratio_at_60pct_zero_no_mask"]
    total = oracle.compressed_bytes(n, 4, nnz)
    assert x.nbytes / total == pytest.approx(32 / (1 + 32 * 0.4), rel=1e-12)


# --------------------------------------------------------------------------
# library-routine second implementation, ragged sizes, both widths
# --------------------------------------------------------------------------
@pytest.mark.parametrize("w", [2, 4])
@pytest.mark.parametrize("n", RAGGED_SIZES)
def test_matches_library_routines(oracle, n, w):
    rng = np.random.default_rng(1000 * w + n)
    for density in (0.0, 0.07, 0.5, 0.93, 1.0):
        words = random_words(rng, n, w, density)
        masks, values, nnz = oracle.compress(words, w)
        lib_masks, lib_values = library_zvc(words)
        assert masks.tolist() == lib_masks.tolist()
        assert values.tobytes() == lib_values.tobytes()
        assert nnz == int(np.count_nonzero(words)) == oracle.count_nonzero(words, w)
        assert sum(bin(int(m)).count("1") for m in masks) == nnz
        stream = oracle.compress_stream(words, w)
        assert stream.size == 4 * ((n + 31) // 32) + w * nnz
        assert stream.tobytes() == lib_masks.astype("<u4").tobytes() + lib_values.tobytes()
        assert oracle.decompress_stream(stream, n, w).tobytes() == words.tobytes()
        assert oracle.decompress(masks, values, n, w).tobytes() == words.tobytes()


def test_single_nonzero_every_position_bruteforce(oracle):
    """One non-zero at each position of a 3-group tensor: mask index, bit
    index and kept value are known by construction."""
    for w, dtype in ((4, np.uint32), (2, np.uint16)):
        n = 70
        for pos in range(n):
            x = np.zeros(n, dtype=dtype)
            x[pos] = pos + 1
            masks, values, nnz = oracle.compress(x, w)
            expect = [0, 0, 0]
            expect[pos // 32] = 1 << (pos % 32)
            assert masks.tolist() == expect
            assert nnz == 1 and values.view(dtype).tolist() == [pos + 1]


def test_decoder_places_values_by_mask_bruteforce(oracle):
    """Decoder alone, on masks written by hand (not produced by the encoder)."""
    masks = np.array([0x80000005, 0x00000002], dtype=np.uint32)
    values = np.array([11, 22, 33, 44], dtype=np.uint32)
    out = oracle.decompress(masks, values, 40, 4).view(np.uint32)
    expect = np.zeros(40, dtype=np.uint32)
    expect[0], expect[2], expect[31], expect[33] = 11, 22, 33, 44
    assert out.tolist() == expect.tolist()
    out16 = oracle.decompress(masks, values.astype(np.uint16), 40, 2).view(np.uint16)
    assert out16.tolist() == expect.tolist()


# --------------------------------------------------------------------------
# invariants of the scheme
# --------------------------------------------------------------------------
def test_special_float_patterns_are_kept(oracle):
    """Zero means the all-zero bit pattern: -0.0, NaN payloads, denormals and
    infinities are non-zero and survive the round trip bit for bit."""
    specials32 = np.array([0x80000000, 0x7FC00000, 0x7F800001, 0xFFC12345, 0x00000001,
                           0x807FFFFF, 0x7F800000, 0xFF800000, 0x00000000, 0x3F800000],
                          dtype=np.uint32)
    x = np.tile(specials32, 13)  # 130 elements, ragged
    masks, values, nnz = oracle.compress(x, 4)
    assert nnz == 13 * 9 == oracle.count_nonzero(x, 4)
    assert oracle.decompress(masks, values, x.size, 4).tobytes() == x.tobytes()
    # as floats: -0.0 == 0.0 compares equal, but it must still be kept
    f = x.view(np.float32)
    assert np.count_nonzero(f == 0.0) == 26 and x.size - nnz == 13
    specials16 = np.array([0x8000, 0x7E00, 0x7C01, 0x0001, 0x83FF, 0x7C00, 0xFC00, 0x0000,
                           0x3C00, 0xFFFF], dtype=np.uint16)
    y = np.tile(specials16, 13)
    masks, values, nnz = oracle.compress(y, 2)
    assert nnz == 13 * 9 == oracle.count_nonzero(y, 2)
    assert oracle.decompress(masks, values, y.size, 2).tobytes() == y.tobytes()


@pytest.mark.parametrize("w", [2, 4])
def test_extremes(oracle, w):
    dtype = np.uint32 if w == 4 else np.uint16
    for n in (32, 64 * 32, 1000, 4097):
        G = (n + 31) // 32
        z = np.zeros(n, dtype=dtype)
        masks, values, nnz = oracle.compress(z, w)
        assert nnz == 0 and values.size == 0 and not masks.any()
        assert oracle.compressed_bytes(n, w, 0) == 4 * G
        if n % 32 == 0:
            assert n * w / (4 * G) == 8 * w  # 32x for fp32, 16x for 16-bit
        ones = np.arange(1, n + 1).astype(dtype)
        ones[ones == 0] = 1
        masks, values, nnz = oracle.compress(ones, w)
        assert nnz == n and values.tobytes() == ones.tobytes()
        tail = n % 32
        expect_last = 0xFFFFFFFF if tail == 0 else (1 << tail) - 1
        assert masks[:-1].tolist() == [0xFFFFFFFF] * (G - 1) and int(masks[-1]) == expect_last
        assert oracle.compressed_bytes(n, w, nnz) == 4 * G + w * n
        if n % 32 == 0 and w == 4:
            assert n * w / oracle.compressed_bytes(n, w, nnz) == pytest.approx(32 / 33)


@pytest.mark.parametrize("w", [2, 4])
def test_ratio_closed_form_on_bernoulli(oracle, w):
    rng = np.random.default_rng(7)
    n = 32 * 20000
    for d in (0.05, 0.2, 0.5, 0.8):
        words = random_words(rng, n, w, d)
        stream = oracle.compress_stream(words, w)
        realised = np.count_nonzero(words) / n
        ratio = n * w / stream.size
        assert ratio == pytest.approx(8 * w / (1 + 8 * w * realised), rel=1e-12)
        assert ratio == pytest.approx(8 * w / (1 + 8 * w * d), rel=0.02)


def test_layout_independence(oracle):
    """Section 5.1 / 7.1: the compressed size depends only on how many values
    are zero, not on where they are: NCHW, NHWC and CHWN orders of one tensor
    compress to the same number of bytes."""
    rng = np.random.default_rng(3)
    x = rng.standard_normal((6, 10, 7, 9)).astype(np.float32)
    x[rng.random(x.shape) < 0.65] = 0.0
    sizes = set()
    for perm in ((0, 1, 2, 3), (0, 2, 3, 1), (1, 2, 3, 0)):
        y = np.ascontiguousarray(x.transpose(perm))
        s = oracle.compress_stream(y, 4)
        sizes.add(s.size)
        assert oracle.decompress_stream(s, y.size, 4).tobytes() == y.tobytes()
    assert len(sizes) == 1


def test_random_byte_soup_round_trip(oracle):
    rng = np.random.default_rng(11)
    for w in (2, 4):
        for n in (1, 77, 5000):
            raw = rng.integers(0, 256, size=n * w, dtype=np.uint8)
            raw[rng.random(n * w) < 0.5] = 0  # many zero bytes, some zero elements
            s = oracle.compress_stream(raw, w)
            assert oracle.decompress_stream(s, n, w).tobytes() == raw.tobytes()


def test_values_preserve_order(oracle):
    x = np.zeros(200, dtype=np.uint32)
    idx = np.array([3, 31, 32, 64, 65, 130, 199])
    x[idx] = idx + 100
    _, values, _ = oracle.compress(x, 4)
    assert values.view(np.uint32).tolist() == (idx + 100).tolist()


def test_bad_width_rejected(oracle):
    with pytest.raises(ValueError):
        oracle.compress(np.zeros(8, dtype=np.uint8), 1)
    with pytest.raises(ValueError):
        oracle.compress_stream(np.zeros(8, dtype=np.uint8), 8)
