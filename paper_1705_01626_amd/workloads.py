"""Seeded synthetic activation tensors shaped like the paper's CNN workloads.

This module only DRAWS inputs.  It contains none of the compression method's
arithmetic (no masks, no packing, no counting) and is the one module that both
the GPU path's tests/bench and the CPU oracle's tests may use, so that both
sides see the same bytes.

The tensors stand in for the ImageNet-trained activations the paper measures
(section 4: roughly half of the first convolution's outputs are zero, deeper
layers are sparser, zeros cluster spatially; section 2.3: NCHW / NHWC / CHWN
memory orders).  Every draw is a pure function of (recipe, shape, seed, device
type); torch's CPU and GPU generators give different streams, so a test
generates once and hands the same bytes to both sides.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, Iterator, List, Optional, Sequence, Tuple

import torch

_TINY32 = 1.1754943508222875e-38  # smallest positive normal fp32


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _abs_normal_nonzero(shape, g: torch.Generator, device) -> torch.Tensor:
    """|N(0,1)| with any exact zero draw replaced by the smallest normal."""
    v = torch.randn(shape, generator=g, device=device, dtype=torch.float32).abs_()
    v.clamp_(min=_TINY32)
    return v


def pre_activation(post: torch.Tensor, seed: int) -> torch.Tensor:
    """A pre-activation tensor whose ReLU is `post` (fp32, a ReLU output): every
    zero of `post` becomes a negative draw -|N(0,1)|, a few of them -0.0 or +0.0;
    positive elements stay as they are.  Stands in for a convolution's output
    before its ReLU layer (section 4)."""
    g = _gen(seed, post.device)
    neg = torch.randn(post.shape, generator=g, device=post.device, dtype=torch.float32).abs_().neg_()
    pick = torch.rand(post.shape, generator=g, device=post.device)
    neg = torch.where(pick < 0.01, torch.zeros_like(neg), neg)          # +0.0
    neg = torch.where(pick > 0.99, -torch.zeros_like(neg), neg)         # -0.0
    return torch.where(post > 0, post, neg)


def relu_gaussian(shape: Sequence[int], density: float, seed: int, device="cpu") -> torch.Tensor:
    """max(0, N(mu, 1)) iid, with mu chosen so that P(x > 0) = density."""
    mu = math.sqrt(2.0) * float(torch.erfinv(torch.tensor(2.0 * density - 1.0, dtype=torch.float64)))
    g = _gen(seed, device)
    x = torch.randn(tuple(shape), generator=g, device=device, dtype=torch.float32)
    x.add_(mu).clamp_(min=0.0)
    return x


def bernoulli_sparse(shape: Sequence[int], density: float, seed: int, device="cpu",
                     chunk_elems: int = 1 << 26) -> torch.Tensor:
    """iid Bernoulli(density) support with |N(0,1)| magnitudes (never exactly 0).

    density = 1.0 gives a tensor with no zero at all.
    """
    g = _gen(seed, device)
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, device=device, dtype=torch.float32)
    for lo in range(0, n, chunk_elems):
        hi = min(n, lo + chunk_elems)
        v = _abs_normal_nonzero((hi - lo,), g, device)
        if density < 1.0:
            keep = torch.rand((hi - lo,), generator=g, device=device, dtype=torch.float32) < density
            v.mul_(keep)
        out[lo:hi] = v
    return out.view(tuple(shape))


def _gaussian_taps(sigma: float, device) -> torch.Tensor:
    radius = int(math.ceil(3.0 * sigma))
    t = torch.arange(-radius, radius + 1, device=device, dtype=torch.float32)
    k = torch.exp(-(t * t) / (2.0 * sigma * sigma))
    return k / k.sum()


def blurred_field(shape: Sequence[int], channel_density: torch.Tensor, seed: int, device="cpu",
                  sigma: float = 2.0, chunk_planes: int = 2048) -> torch.Tensor:
    """Spatially clustered sparsity for an (N, C, H, W) tensor.

    Per (n, c) plane an N(0,1) field is blurred with a separable Gaussian of
    `sigma` pixels (zero padded) and the plane keeps the round(d_c * H * W)
    positions with the largest blurred value, d_c = channel_density[c].
    Kept positions get |N(0,1)| magnitudes; the rest are exactly 0.
    """
    N, C, H, W = (int(s) for s in shape)
    g = _gen(seed, device)
    taps = _gaussian_taps(sigma, device)
    r = (taps.numel() - 1) // 2
    kx = taps.view(1, 1, 1, -1)
    ky = taps.view(1, 1, -1, 1)
    dens = channel_density.to(device=device, dtype=torch.float32)
    plane_d = dens.repeat(N)  # plane p = n * C + c  ->  density of channel c
    keep_count = torch.round(plane_d * (H * W)).to(torch.int64).clamp_(0, H * W)
    out = torch.empty((N * C, H * W), device=device, dtype=torch.float32)
    for lo in range(0, N * C, chunk_planes):
        hi = min(N * C, lo + chunk_planes)
        f = torch.randn((hi - lo, 1, H, W), generator=g, device=device, dtype=torch.float32)
        f = torch.nn.functional.conv2d(f, kx, padding=(0, r))
        f = torch.nn.functional.conv2d(f, ky, padding=(r, 0))
        f = f.view(hi - lo, H * W)
        # threshold = the keep_count-th largest blurred value of each plane
        srt, _ = torch.sort(f, dim=1, descending=True)
        kc = keep_count[lo:hi]
        idx = (kc - 1).clamp_(min=0).view(-1, 1)
        thr = torch.gather(srt, 1, idx)
        keep = (f >= thr) & (kc.view(-1, 1) > 0)
        v = _abs_normal_nonzero((hi - lo, H * W), g, device)
        out[lo:hi] = v * keep
    return out.view(N, C, H, W)


def uniform_channel_density(channels: int, lo: float, hi: float, seed: int) -> torch.Tensor:
    """One density per channel drawn U[lo, hi] (CPU generator: device independent)."""
    g = _gen(seed, "cpu")
    return lo + (hi - lo) * torch.rand((channels,), generator=g, dtype=torch.float32)


# ----------------------------------------------------------------------------
# The five benchmark workloads.  `batch` overrides the leading dimension so the
# same recipe can be drawn at a size a CPU oracle finishes in seconds.
# ----------------------------------------------------------------------------

def conv_small(seed: int = 0, device="cpu", batch: int = 8) -> torch.Tensor:
    """Workload 0: fp32 NCHW 8x64x56x56, ReLU of a shifted Gaussian, 40 % non-zero."""
    return relu_gaussian((batch, 64, 56, 56), 0.4, seed, device)


def conv1_style(seed: int = 0, device="cpu", batch: int = 256) -> torch.Tensor:
    """Workload 1: fp32 NCHW 256x96x55x55 (first-convolution output of an
    AlexNet-sized network), per-channel density U[0.1, 0.9], blurred-field support."""
    dens = uniform_channel_density(96, 0.1, 0.9, seed + 1)
    return blurred_field((batch, 96, 55, 55), dens, seed, device)


DENSITY_SWEEP = (0.05, 0.2, 0.5, 0.8, 1.0)


def density_sweep(density: float, seed: int = 0, device="cpu", batch: int = 64) -> torch.Tensor:
    """Workload 2: fp32 NCHW 64x64x224x224, iid Bernoulli(density) support."""
    return bernoulli_sparse((batch, 64, 224, 224), density, seed, device)


@dataclass(frozen=True)
class LayerSpec:
    name: str
    shape: Tuple[int, ...]
    density: float


def vgg_offload_stream(batch: int = 64) -> List[LayerSpec]:
    """Workload 3: the 16 ReLU outputs of a VGG-16-style network, densities
    falling linearly from 0.6 (first layer) to 0.1 (last)."""
    conv = [(64, 224), (64, 224), (128, 112), (128, 112), (256, 56), (256, 56), (256, 56),
            (512, 28), (512, 28), (512, 28), (512, 14), (512, 14), (512, 14)]
    shapes: List[Tuple[int, ...]] = [(batch, c, s, s) for c, s in conv]
    shapes += [(batch, 4096), (batch, 4096), (batch, 1000)]
    specs = []
    for i, shp in enumerate(shapes):
        d = 0.6 - 0.5 * i / 15.0
        kind = "conv" if len(shp) == 4 else "fc"
        specs.append(LayerSpec("%s%02d" % (kind, i), shp, d))
    return specs


def vgg_layer(spec: LayerSpec, index: int, seed: int = 0, device="cpu") -> torch.Tensor:
    return bernoulli_sparse(spec.shape, spec.density, seed * 1000 + index, device)


LAYOUT_VARIANTS = ("fp32_nchw", "fp32_nhwc", "fp32_chwn", "fp16_nchw", "bf16_nchw")


def layout_variants(seed: int = 0, device="cpu", batch: int = 128,
                    shape_tail: Tuple[int, int, int] = (256, 28, 28)) -> Dict[str, torch.Tensor]:
    """Workload 4: one logical 128x256x28x28 tensor at 30 % blurred-field
    density, stored as fp32 in NCHW / NHWC / CHWN memory order and as fp16 /
    bf16 (NCHW).  The 16-bit variants are converted from the fp32 tensor first;
    whatever is zero after conversion is what the codec sees."""
    C, H, W = shape_tail
    dens = torch.full((C,), 0.3)
    x = blurred_field((batch, C, H, W), dens, seed, device)
    return {
        "fp32_nchw": x,
        "fp32_nhwc": x.permute(0, 2, 3, 1).contiguous(),
        "fp32_chwn": x.permute(1, 2, 3, 0).contiguous(),
        "fp16_nchw": x.to(torch.float16),
        "bf16_nchw": x.to(torch.bfloat16),
    }
