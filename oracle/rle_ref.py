"""Zero-run run-length encoding, sizes only: the layout-sensitive scheme the
paper compares ZVC against (section 5.1 "Run-length encoding compression",
section 7.1 and its figure on compression ratio by data layout).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/: plain numpy, no GPU.

The paper does not give its RLE format.  This one is the plainest zero-run
code: inside every window of `window_bytes` of uncompressed data (4 KB in the
paper's comparison) the elements are cut into records, each a run of zero
elements followed by a run of non-zero elements (either may be empty, not
both); a record costs a 16-bit zero count, a 16-bit literal count and the
literals themselves.  Runs do not cross windows.  Only the size is computed.
"""
from __future__ import annotations

import numpy as np


def rle_compressed_bytes(words: np.ndarray, window_bytes: int = 4096) -> int:
    """words: uint16/uint32 element bit patterns (flat).  Returns the RLE size in bytes."""
    words = np.ascontiguousarray(words).reshape(-1)
    w = words.dtype.itemsize
    per = window_bytes // w
    total = 0
    for lo in range(0, words.size, per):
        nz = words[lo: lo + per] != 0
        # a record starts at the window's start and wherever a zero follows a non-zero
        starts = 1 + int(np.count_nonzero(nz[:-1] & ~nz[1:]))
        total += 4 * starts + w * int(np.count_nonzero(nz))
    return total


def zvc_compressed_bytes(words: np.ndarray) -> int:
    """4 * ceil(n / 32) + w * nnz (section 5.1), for the comparison table."""
    words = np.ascontiguousarray(words).reshape(-1)
    return 4 * ((words.size + 31) // 32) + words.dtype.itemsize * int(np.count_nonzero(words))
