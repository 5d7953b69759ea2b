"""Seeded random sweep of the HIP path against the CPU oracle: random sizes,
element widths, pointer offsets, sparsity structure (iid, runs of zeros, dense
and empty stretches) and entry points (plain, fused ReLU, bounded, windowed),
one workspace reused throughout.  Bit-exact comparison."""
import os

import numpy as np
import pytest
import torch

from paper_1705_01626_amd import zvc
from tests.gpu_util import raw_bytes, say

pytestmark = pytest.mark.gpu
DEV = "cuda"
DTYPES = {4: torch.int32, 2: torch.int16}
CASES = int(os.environ.get("ZVC_SWEEP_CASES", "60"))      # more cases for a longer run
SEED = int(os.environ.get("ZVC_SWEEP_SEED", "20240607"))
MAX_N = int(os.environ.get("ZVC_SWEEP_MAX_N", str(5 << 20)))   # default reaches the 16 and 32 KB tile kernels


def structured_words(rng, n, w):
    """Random words whose zeros come iid, in runs, or in long empty/dense stretches."""
    hi = 2 ** (8 * w - 1)
    x = rng.integers(-hi, hi, size=n, dtype=np.int64)
    kind = rng.integers(0, 4)
    if kind == 0:                                   # iid
        x[rng.random(n) < rng.random()] = 0
    elif kind == 1:                                 # runs of zeros and of values, geometric lengths
        pos, keep = 0, bool(rng.integers(0, 2))
        mean = int(rng.integers(8, 400))
        while pos < n:
            run = int(rng.geometric(1.0 / mean))
            if not keep:
                x[pos:pos + run] = 0
            pos, keep = pos + run, not keep
    elif kind == 2:                                 # empty and dense stretches of tile size and more
        step = int(rng.integers(1000, 70000))
        for lo in range(0, n, step):
            mode = rng.integers(0, 3)
            if mode == 0:
                x[lo:lo + step] = 0
            elif mode == 1:
                x[lo:lo + step][rng.random(min(step, n - lo)) < 0.5] = 0
    else:                                           # nearly empty
        x[rng.random(n) < 0.999] = 0
    x[rng.random(n) < 0.01] = -hi                   # the pattern of -0.0
    return x.astype({4: np.int32, 2: np.int16}[w])


def test_random_sweep(oracle):
    rng = np.random.default_rng(SEED)
    ws = zvc.new_workspace(MAX_N + 64, 4, DEV)
    for case in range(CASES):
        w = int(rng.choice([2, 4]))
        n = int(rng.integers(1, MAX_N)) if case % 5 else int(rng.integers(1, 5000))
        offset = int(rng.choice([0, 0, 4, 8, 1, 3])) if w == 4 else int(rng.choice([0, 0, 8, 16, 1, 5]))
        host_words = structured_words(rng, n, w)
        base = torch.zeros(n + 32, dtype=DTYPES[w], device=DEV)
        x = base[offset:offset + n]
        x.copy_(torch.from_numpy(host_words))
        host = raw_bytes(x)
        mode = ("plain", "relu", "bounded", "windowed")[case % 4]
        say("sweep case %d: mode=%s n=%d w=%d offset=%d" % (case, mode, n, w, offset))
        d_bytes = torch.full((1,), -1, dtype=torch.int64, device=DEV)
        out_base = torch.full((n + 32,), 0x55, dtype=DTYPES[w], device=DEV)
        out = out_base[offset:offset + n]
        if mode in ("plain", "relu"):
            expect = oracle.relu_compress_stream(host, w) if mode == "relu" else oracle.compress_stream(host, w)
            comp = zvc.new_compressed_buffer(n, w, DEV)
            (zvc.zvc_relu_compress if mode == "relu" else zvc.zvc_compress)(x, comp, d_bytes, ws)
            assert int(d_bytes.item()) == expect.size
            assert np.array_equal(comp[:expect.size].cpu().numpy(), expect)
            zvc.zvc_decompress(comp, expect.size, out, ws)
            torch.cuda.synchronize()
            want = oracle.relu(host, w) if mode == "relu" else host
            assert np.array_equal(raw_bytes(out), want)
        elif mode == "bounded":
            expect = oracle.compress_stream(host, w)
            comp = torch.full((expect.size + 256,), 0xA7, dtype=torch.uint8, device=DEV)
            zvc.zvc_compress_bounded(x, comp, d_bytes, ws, out_cap=expect.size)
            assert int(d_bytes.item()) == expect.size
            got = comp.cpu().numpy()
            assert np.array_equal(got[:expect.size], expect) and (got[expect.size:] == 0xA7).all()
            zvc.zvc_decompress(comp, expect.size, out, ws)
            torch.cuda.synchronize()
            assert np.array_equal(raw_bytes(out), host)
        else:
            window = 1024 << int(rng.integers(0, 7))            # 1 KB .. 64 KB
            per = window // w
            expect, table = oracle.window_compress(host, w, per)
            windows = zvc.zvc_window_count(n, w, window)
            comp = zvc.new_compressed_buffer(n, w, DEV)
            offsets = torch.zeros(windows + 1, dtype=torch.int64, device=DEV)
            zvc.zvc_window_compress(x, comp, offsets, d_bytes, ws, window_bytes=window)
            assert int(d_bytes.item()) == expect.size
            assert np.array_equal(comp[:expect.size].cpu().numpy(), expect)
            assert offsets.cpu().numpy().astype(np.uint64).tolist() == table.tolist()
            first = int(rng.integers(0, windows))
            count = int(rng.integers(1, windows - first + 1))
            part_elems = min(n - first * per, count * per)
            part = out[:part_elems]
            zvc.zvc_window_decompress(comp, expect.size, offsets, n, first, count, part, window_bytes=window)
            torch.cuda.synchronize()
            assert np.array_equal(raw_bytes(part), host[first * per * w:(first * per + part_elems) * w])
        # the elements around the output range are untouched
        assert int((out_base[:offset] != 0x55).sum()) == 0
        assert int((out_base[offset + n:] != 0x55).sum()) == 0
