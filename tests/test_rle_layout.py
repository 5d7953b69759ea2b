"""ZVC against a zero-run RLE across data layouts (the shape of the paper's
compression-ratio-by-layout figure, section 7.1): ZVC's size depends only on
how many elements are non-zero, RLE's on how they are arranged.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import rle_ref
from paper_1705_01626_amd import workloads


def brute_force_rle_bytes(words, per):
    """Records counted by walking the elements one by one."""
    total, w = 0, words.dtype.itemsize
    for lo in range(0, len(words), per):
        win = words[lo: lo + per]
        i = 0
        while i < len(win):
            zeros = 0
            while i < len(win) and win[i] == 0:
                zeros += 1; i += 1
            lits = 0
            while i < len(win) and win[i] != 0:
                lits += 1; i += 1
            total += 4 + w * lits
    return total


def test_rle_hand_cases():
    z = np.zeros(1024, dtype=np.uint32)
    assert rle_ref.rle_compressed_bytes(z) == 4                       # one record: 1024 zeros
    d = np.ones(1024, dtype=np.uint32)
    assert rle_ref.rle_compressed_bytes(d) == 4 + 4096                # one record: 1024 literals
    alt = np.tile(np.array([0, 1], dtype=np.uint32), 512)
    assert rle_ref.rle_compressed_bytes(alt) == 512 * (4 + 4)         # worst case: a record per pair
    two = np.zeros(2048, dtype=np.uint32)
    assert rle_ref.rle_compressed_bytes(two) == 8                     # runs stop at the window border
    x = np.array([5, 0, 0, 7, 7, 0], dtype=np.uint32)
    assert rle_ref.rle_compressed_bytes(x) == (4 + 4) + (4 + 8) + 4


@pytest.mark.parametrize("w", [2, 4])
def test_rle_matches_brute_force(w):
    rng = np.random.default_rng(w)
    dtype = np.uint32 if w == 4 else np.uint16
    for n in (0, 1, 1023, 1024, 1025, 5000):
        for density in (0.0, 0.1, 0.5, 0.9, 1.0):
            words = (rng.integers(1, 1000, n) * (rng.random(n) < density)).astype(dtype)
            assert rle_ref.rle_compressed_bytes(words) == brute_force_rle_bytes(words, 4096 // w)


def test_zvc_is_layout_independent_and_rle_is_not(oracle):
    """One logical 16x64x28x28 blurred-field tensor at 30 % density in three memory orders."""
    variants = workloads.layout_variants(seed=0, device="cpu", batch=16, shape_tail=(64, 28, 28))
    sizes = {}
    for name in ("fp32_nchw", "fp32_nhwc", "fp32_chwn"):
        words = variants[name].contiguous().view(torch.int32).numpy().view(np.uint32).reshape(-1)
        zvc = rle_ref.zvc_compressed_bytes(words)
        assert zvc == oracle.compress_stream(words, 4).size             # the formula is the oracle's size
        sizes[name] = (zvc, rle_ref.rle_compressed_bytes(words), words.nbytes)
    zvc_sizes = {v[0] for v in sizes.values()}
    assert len(zvc_sizes) == 1                                           # ZVC does not care where the zeros are
    ratio = {k: v[2] / v[1] for k, v in sizes.items()}
    # zeros cluster along the image rows, which only NCHW keeps contiguous
    assert ratio["fp32_nchw"] > 1.15 * ratio["fp32_nhwc"]
    assert ratio["fp32_nchw"] > 1.15 * ratio["fp32_chwn"]
    zvc_ratio = sizes["fp32_nchw"][2] / sizes["fp32_nchw"][0]
    assert zvc_ratio > ratio["fp32_nhwc"] and zvc_ratio > ratio["fp32_chwn"]


@pytest.mark.gpu
def test_ratio_by_layout_at_full_size(oracle):
    """The layout comparison at the full 128x256x28x28 size (section 7.1, the
    compression-ratio-by-layout figure: ZVC compresses equally well however the
    zeros are arranged, a run-length code does not).  ZVC sizes come from the GPU
    (zvc_compressed_size), RLE sizes from the numpy reference; prints the table."""
    from paper_1705_01626_amd import zvc
    from tests.gpu_util import say
    variants = workloads.layout_variants(seed=0, device="cuda")
    rows = {}
    for name in ("fp32_nchw", "fp32_nhwc", "fp32_chwn", "fp16_nchw", "bf16_nchw"):
        x = variants[name].contiguous()
        n, w = x.numel(), x.element_size()
        assert n == 128 * 256 * 28 * 28
        ws = zvc.new_workspace(n, w, x.device)
        d_bytes = torch.zeros(1, dtype=torch.int64, device=x.device)
        say("ratio by layout: %s" % name)
        zvc.zvc_compressed_size(x, d_bytes, ws)
        gpu_bytes = int(d_bytes.item())
        words = x.view(torch.int32 if w == 4 else torch.int16).cpu().numpy().view(np.uint32 if w == 4 else np.uint16).reshape(-1)
        assert gpu_bytes == rle_ref.zvc_compressed_bytes(words)           # the size formula on the host
        rows[name] = (n * w, gpu_bytes, rle_ref.rle_compressed_bytes(words, 4096))
    print("\n[layout-ratio] layout      bytes        ZVC bytes   ZVC ratio   RLE bytes (4 KB windows)   RLE ratio")
    for name, (ub, zb, rb) in rows.items():
        print("[layout-ratio] %-10s %11d %11d   %8.3f   %11d                %8.3f" % (name, ub, zb, ub / zb, rb, ub / rb))
    zvc_fp32 = {rows[k][1] for k in ("fp32_nchw", "fp32_nhwc", "fp32_chwn")}
    assert len(zvc_fp32) == 1                                             # layout independent, to the byte
    rle = {k: rows[k][0] / rows[k][2] for k in rows}
    zr = rows["fp32_nchw"][0] / rows["fp32_nchw"][1]
    assert rle["fp32_nchw"] > 1.15 * rle["fp32_nhwc"] and rle["fp32_nchw"] > 1.15 * rle["fp32_chwn"]
    assert zr > rle["fp32_nhwc"] and zr > rle["fp32_chwn"]
