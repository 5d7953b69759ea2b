"""Pins for the oracle's paper-order windowed stream.  No GPU needed.

Checked against hand-worked byte streams, an independent parser written in
plain Python that walks a stream the way the paper describes its decoder
(read a mask, its popcount says how many words follow), the planar stream of
the same input (same masks, same values, same byte count), and the properties
the window table must have.
"""
import numpy as np
import pytest

from tests.golden_cases import load_window_cases
from tests.test_oracle import library_zvc, random_words


def walk_stream(stream: bytes, n: int, w: int):
    """Serial walk: mask, then popcount(mask) elements, until n elements are covered."""
    masks, values, pos, covered = [], [], 0, 0
    while covered < n:
        m = int.from_bytes(stream[pos:pos + 4], "little")
        pos += 4
        masks.append(m)
        k = bin(m).count("1")
        values.append(stream[pos:pos + k * w])
        pos += k * w
        covered += 32
    return masks, b"".join(values), pos


@pytest.mark.parametrize("case", load_window_cases(), ids=lambda c: c["name"])
def test_window_handbuilt_cases(oracle, case):
    stream, offsets = oracle.window_compress(case["in"], case["w"], case["window"])
    assert stream.tobytes() == case["stream"].tobytes()
    assert offsets.tolist() == case["offsets"].tolist()
    windows = len(case["offsets"]) - 1
    back = oracle.window_decompress(stream, offsets, case["n"], case["w"], case["window"], 0, windows)
    assert back.tobytes() == case["in"].tobytes()


@pytest.mark.parametrize("w", [2, 4])
@pytest.mark.parametrize("n", [0, 1, 31, 32, 33, 1023, 1024, 1025, 4097, 12345])
def test_window_stream_holds_the_planar_masks_and_values(oracle, n, w):
    rng = np.random.default_rng(77 * n + w)
    for density in (0.0, 0.3, 1.0):
        words = random_words(rng, n, w, density)
        for window in (32, 1024, 2048):
            stream, offsets = oracle.window_compress(words, w, window)
            masks, values, end = walk_stream(stream.tobytes(), n, w)
            lib_masks, lib_values = library_zvc(words)
            assert masks == lib_masks.tolist()
            assert values == lib_values.tobytes()
            assert end == stream.size == 4 * ((n + 31) // 32) + w * int(np.count_nonzero(words))
            assert stream.size == oracle.compress_stream(words, w).size      # window size costs nothing
            # the table: cumulative bytes of whole windows
            K = (n + window - 1) // window
            assert offsets.size == K + 1 and offsets[0] == 0 and offsets[-1] == stream.size
            for k in range(K):
                chunk = words[k * window:(k + 1) * window]
                assert offsets[k + 1] - offsets[k] == 4 * ((chunk.size + 31) // 32) + w * int(np.count_nonzero(chunk))


@pytest.mark.parametrize("w", [2, 4])
def test_any_window_range_decodes_on_its_own(oracle, w):
    rng = np.random.default_rng(5 + w)
    n, window = 10 * 1024 + 77, 1024
    words = random_words(rng, n, w, 0.4)
    stream, offsets = oracle.window_compress(words, w, window)
    K = offsets.size - 1
    for first, count in ((0, K), (0, 1), (3, 4), (K - 1, 1), (K, 0), (5, 0)):
        got = oracle.window_decompress(stream, offsets, n, w, window, first, count)
        assert got.tobytes() == words[first * window:(first + count) * window].tobytes()
    # a window decodes from its own bytes alone: damage everything else
    k = 4
    lo, hi = int(offsets[k]), int(offsets[k + 1])
    damaged = np.full_like(stream, 0x5A)
    damaged[lo:hi] = stream[lo:hi]
    got = oracle.window_decompress(damaged, offsets, n, w, window, k, 1)
    assert got.tobytes() == words[k * window:(k + 1) * window].tobytes()


def test_window_special_patterns_round_trip(oracle):
    """-0.0, NaN, denormals and infinities are kept bit for bit; all-zero and dense windows."""
    specials = np.array([0x80000000, 0x7FC00000, 0x00000001, 0xFF800000, 0, 0, 0x3F800000, 0] * 300, dtype=np.uint32)
    stream, offsets = oracle.window_compress(specials, 4, 1024)
    assert oracle.window_decompress(stream, offsets, specials.size, 4, 1024, 0, offsets.size - 1).tobytes() == specials.tobytes()
    zeros = np.zeros(2048, dtype=np.uint32)
    stream, offsets = oracle.window_compress(zeros, 4, 1024)
    assert stream.size == 4 * 64 and not stream.any() and offsets.tolist() == [0, 128, 256]
    dense = np.arange(1, 2049, dtype=np.uint32)
    stream, offsets = oracle.window_compress(dense, 4, 1024)
    assert offsets.tolist() == [0, 1024 * 4 + 128, 2 * (1024 * 4 + 128)]


def test_window_bad_arguments_rejected(oracle):
    x = np.zeros(64, dtype=np.uint32)
    for window in (0, 31, 48):
        with pytest.raises(ValueError):
            oracle.window_compress(x, 4, window)
    with pytest.raises(ValueError):
        oracle.window_compress(x, 3, 32)
    stream, offsets = oracle.window_compress(x, 4, 32)
    with pytest.raises(ValueError):
        oracle.window_decompress(stream, offsets, 64, 4, 32, 1, 2)    # past the last window
