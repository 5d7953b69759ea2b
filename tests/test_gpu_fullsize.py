"""GPU parity at the full sizes of the benchmark workloads, in the launch
configuration bench.py times (tile sizes are chosen from the tensor size, so
only full-size tensors reach the large-tile kernels).  The oracle handles
these sizes in seconds, so the comparison is still element by element."""
import numpy as np
import pytest
import torch

from paper_1705_01626_amd import workloads, zvc
from tests.gpu_util import assert_parity, raw_bytes, say

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _density(res, x):
    n, w = x.numel(), x.element_size()
    return (res["bytes"] - 4 * ((n + 31) // 32)) / w / n


def test_conv1_style_full(oracle):
    """fp32 256x96x55x55, per-channel density U[0.1,0.9], blurred-field support."""
    x = workloads.conv1_style(seed=0, device=DEV)
    assert x.numel() == 74342400
    res = assert_parity(x, oracle, "conv1_style full")
    assert 0.45 < _density(res, x) < 0.56
    say("self-help events: %d" % zvc.zvc_workspace_self_help_count(res["ws"]))


@pytest.mark.parametrize("density", workloads.DENSITY_SWEEP)
def test_density_sweep_full(oracle, density):
    """fp32 64x64x224x224 at each density of the sweep; ratio follows 32/(1+32d)."""
    x = workloads.density_sweep(density, seed=0, device=DEV)
    assert x.numel() == 205520896
    res = assert_parity(x, oracle, "sweep d=%.2f full" % density)
    d = _density(res, x)
    assert abs(d - density) < 2e-3
    ratio = x.numel() * 4 / res["bytes"]
    assert ratio == pytest.approx(32 / (1 + 32 * d), rel=1e-9)
    if density == 1.0:
        assert res["bytes"] == zvc.zvc_max_compressed_bytes(x.numel(), 4)
    del x, res
    torch.cuda.empty_cache()


def test_layout_variants_full(oracle):
    """128x256x28x28 at 30 % blurred-field density: NCHW/NHWC/CHWN give identical
    sizes (section 5.1: ZVC does not care where the zeros are); fp16 and bf16."""
    variants = workloads.layout_variants(seed=0, device=DEV)
    sizes = {}
    for name, t in variants.items():
        assert t.numel() == 25690112
        sizes[name] = assert_parity(t, oracle, "layout %s full" % name)["bytes"]
    assert sizes["fp32_nchw"] == sizes["fp32_nhwc"] == sizes["fp32_chwn"]
    n = 25690112
    assert abs((sizes["fp32_nchw"] - n // 8) / 4 / n - 0.3) < 0.01
    # bf16 keeps every non-zero of the fp32 tensor; fp16 may flush a few tiny ones to zero
    assert (sizes["bf16_nchw"] - n // 8) // 2 == (sizes["fp32_nchw"] - n // 8) // 4
    assert (sizes["fp16_nchw"] - n // 8) // 2 <= (sizes["fp32_nchw"] - n // 8) // 4


def test_vgg_offload_stream_full(oracle):
    """The 16 ReLU outputs of a VGG-16-style network at batch 64, each compressed,
    copied to pinned host memory, copied back and decompressed on two streams.
    Host-side bytes are compared with the oracle, the round trip with the input."""
    specs = workloads.vgg_offload_stream()
    assert len(specs) == 16
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    biggest = max(int(np.prod(s.shape)) for s in specs)
    cap = zvc.zvc_max_compressed_bytes(biggest, 4)
    stage = torch.empty(cap, dtype=torch.uint8, device=DEV)
    h_pinned = torch.empty(cap, dtype=torch.uint8, pin_memory=True)
    h_bytes = torch.zeros(1, dtype=torch.int64, pin_memory=True)
    ws = zvc.new_workspace(biggest, 4, DEV)
    total_in = total_out = 0
    for i, spec in enumerate(specs):
        x = workloads.vgg_layer(spec, i, seed=0, device=DEV)
        n = x.numel()
        torch.cuda.synchronize()
        say("vgg layer %d %s n=%d d=%.3f" % (i, spec.name, n, spec.density))
        nbytes = zvc.zvc_offload(x, stage, h_pinned, h_bytes, ws, compute, copy)
        copy.synchronize()
        expect = oracle.compress_stream(raw_bytes(x), 4)
        assert nbytes == expect.size
        assert np.array_equal(h_pinned[:nbytes].numpy(), expect)
        stage.zero_()
        out = torch.empty_like(x)
        torch.cuda.synchronize()
        zvc.zvc_prefetch(h_pinned, nbytes, stage, out, ws, copy, compute)
        compute.synchronize()
        assert torch.equal(out, x)
        d = (nbytes - 4 * ((n + 31) // 32)) / 4 / n
        assert abs(d - spec.density) < 0.01
        total_in += n * 4
        total_out += nbytes
        del x, out
    assert total_in == 3470518272
    # size-weighted ratio of the whole stream (densities 0.6 -> 0.1)
    assert 1.7 < total_in / total_out < 2.0
