"""The paper's bandwidth model of a compressing offload, as host arithmetic.

Section 6 ("Effect of cDMA on memory bandwidth"): a layer whose activations
compress by `ratio` keeps a link of `link` GB/s busy only if the compressor
reads GPU memory at COMP_BW = ratio x link.  When that exceeds the memory
bandwidth the compressor may use (DRAM_BW), the layer's transfer time grows by
COMP_BW / DRAM_BW.  The same reasoning with a software compressor: the link is
fed by kernels that run on the compute stream, and the copy of a tensor can
start only when its compression has finished and the previous copy is done.

Nothing here touches the GPU; bench.py feeds it measured kernel times and
copy rates and prints the prediction beside the measured pipeline.
"""
from __future__ import annotations

from typing import Dict, List, Sequence


def comp_bw(ratio: float, link_gbps: float) -> float:
    """Memory bandwidth (GB/s) the compressor must read at to saturate the link."""
    return ratio * link_gbps


def slowdown(ratio: float, link_gbps: float, dram_gbps: float) -> float:
    """Factor by which a layer's transfer time grows when the compressor cannot be
    fed fast enough: max(1, COMP_BW / DRAM_BW)."""
    return max(1.0, comp_bw(ratio, link_gbps) / dram_gbps)


def transfer_seconds(uncompressed_bytes: float, ratio: float, link_gbps: float,
                     dram_gbps: float) -> float:
    """Transfer time of one layer under the model: compressed bytes over the link,
    inflated by the slowdown factor.  Equals max(compressed / link, uncompressed / DRAM_BW)."""
    compressed = uncompressed_bytes / ratio
    return compressed / (link_gbps * 1e9) * slowdown(ratio, link_gbps, dram_gbps)


def offload_seconds(layers: Sequence[Dict[str, float]], link_gbps: float, dram_gbps: float) -> float:
    """Sum over layers ({"bytes", "ratio"}) of the model's transfer times (hardware
    compressor in the copy path: the transfers simply follow one another)."""
    return sum(transfer_seconds(l["bytes"], l["ratio"], link_gbps, dram_gbps) for l in layers)


def two_stream_pipeline_seconds(compute_s: Sequence[float], copy_s: Sequence[float],
                                host_gap_s: float = 0.0) -> float:
    """Software compressor: tensor i is compressed on one stream (compute_s[i], one
    after the other, plus host_gap_s per tensor for the size read-back) and copied
    on another (copy_s[i]); a copy starts when its tensor is compressed and the
    previous copy is done.  Returns the time at which the last copy ends."""
    done_compute = done_copy = 0.0
    for tc, tx in zip(compute_s, copy_s):
        done_compute += tc + host_gap_s
        done_copy = max(done_compute, done_copy) + tx
    return done_copy


def predict(layers: Sequence[Dict[str, float]], link_gbps: float, host_gap_s: float = 0.0) -> Dict[str, float]:
    """layers: {"bytes", "compressed_bytes", "compress_s"} per tensor, in offload order.
    Returns the predicted offload time of the two-stream pipeline, the time of the
    same copies uncompressed, and how hard the codec works while the link is busy."""
    copy_s = [l["compressed_bytes"] / (link_gbps * 1e9) for l in layers]
    compute_s = [l["compress_s"] for l in layers]
    total = two_stream_pipeline_seconds(compute_s, copy_s, host_gap_s)
    plain = sum(l["bytes"] for l in layers) / (link_gbps * 1e9)
    needed = [comp_bw(l["bytes"] / l["compressed_bytes"], link_gbps) for l in layers]
    have = [l["bytes"] / l["compress_s"] / 1e9 for l in layers]
    return {
        "offload_s": total,
        "uncompressed_s": plain,
        "speedup": plain / total,
        "link_bound_s": sum(copy_s),
        "compute_stream_s": sum(compute_s) + host_gap_s * len(layers),
        # section 6: the compressor must read at COMP_BW to keep the link busy
        "max_comp_bw_needed_gbps": max(needed),
        "min_encoder_read_gbps": min(have),
        "layers_that_starve_the_link": sum(1 for n, h in zip(needed, have) if n > h),
        # memory traffic of the codec averaged over the transfer (read input + write stream)
        "avg_codec_hbm_gbps": sum(l["bytes"] + l["compressed_bytes"] for l in layers) / total / 1e9,
    }
