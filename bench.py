#!/usr/bin/env python3
"""Benchmark of the ZVC hot path on one MI355X.

One "step" is one pass of the whole path over one tensor that is already
resident in HBM: zvc_compress (zero test, masks, per-tile counts, device-wide
scan, compaction, size) followed by zvc_decompress (mask scan, expand) of the
result.  `value` counts the uncompressed bytes that go through the codec per
second: each step pushes n*w bytes through compression and n*w bytes through
decompression, so value = 2*n*w / step time (the per-direction rates are
reported beside it).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Prints ONE JSON line.  Only one GPU is used; --gpus above 1 is refused.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak

WORKLOADS = ("conv_small", "conv1_style", "sweep_0.05", "sweep_0.2", "sweep_0.5", "sweep_0.8",
             "sweep_1.0", "layout_fp32_nchw", "layout_fp32_nhwc", "layout_fp32_chwn",
             "layout_fp16_nchw", "layout_bf16_nchw")


def make_workload(name: str, seed: int, device):
    from paper_1705_01626_amd import workloads
    if name == "conv_small":
        return workloads.conv_small(seed, device), "fp32 NCHW 8x64x56x56, relu(N(mu,1)), 40% non-zero"
    if name == "conv1_style":
        return (workloads.conv1_style(seed, device),
                "fp32 NCHW 256x96x55x55 conv1-style, per-channel density U[0.1,0.9], blurred-field support")
    if name.startswith("sweep_"):
        d = float(name.split("_")[1])
        return (workloads.density_sweep(d, seed, device),
                "fp32 NCHW 64x64x224x224, iid Bernoulli(%.2f) support" % d)
    if name.startswith("layout_"):
        key = name[len("layout_"):]
        return (workloads.layout_variants(seed, device)[key],
                "128x256x28x28 blurred-field 30%% density, %s" % key)
    raise SystemExit("unknown workload %r (choose from %s)" % (name, ", ".join(WORKLOADS)))


def event_timed(fn, reps: int, torch) -> float:
    """Average milliseconds per call of `fn` over `reps` back-to-back launches,
    measured with HIP events recorded on the stream the kernels run on."""
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(reps):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / reps


def cpu_baseline(host_bytes, n: int, w: int, budget_s: float = 10.0, relu: bool = False,
                 windowed: bool = False):
    """The oracle as it stands, single thread, on the same bytes: whole-tensor
    compress + decompress round trips until about `budget_s` seconds are spent.
    With `relu` the encoder is the oracle's fused ReLU + ZVC (ReLU into a
    temporary, then the plain encoder)."""
    import numpy as np
    from oracle import zvc_ref
    lib = zvc_ref.load()
    groups = (n + 31) // 32
    comp = np.zeros(4 * groups + n * w + 16, dtype=np.uint8)
    back = np.zeros(n * w + 16, dtype=np.uint8)
    vp = ctypes.c_void_p
    reps, spent, best = 0, 0.0, None
    while reps < 1 or (spent < budget_s and reps < 50):
        t0 = time.perf_counter()
        if windowed:
            per = 1024 // w
            windows = (n + per - 1) // per
            offsets = np.zeros(windows + 1, dtype=np.uint64)
            lib.zvc_ref_window_compress(vp(host_bytes.ctypes.data), n, w, per, vp(comp.ctypes.data),
                                        vp(offsets.ctypes.data))
            lib.zvc_ref_window_decompress(vp(comp.ctypes.data), vp(offsets.ctypes.data), n, w, per, 0,
                                          windows, vp(back.ctypes.data))
        else:
            encode = lib.zvc_ref_relu_compress_stream if relu else lib.zvc_ref_compress_stream
            encode(vp(host_bytes.ctypes.data), n, w, vp(comp.ctypes.data))
            lib.zvc_ref_decompress_stream(vp(comp.ctypes.data), n, w, vp(back.ctypes.data))
        dt = time.perf_counter() - t0
        spent += dt
        reps += 1
        best = dt if best is None else min(best, dt)
    if relu:
        from oracle import zvc_ref as ref
        assert np.array_equal(back[: n * w], ref.relu(host_bytes[: n * w], w))
    else:
        assert np.array_equal(back[: n * w], host_bytes[: n * w])
    return {"value": round(2.0 * n * w / best / 1e9, 4), "unit": "GB/s", "cores": 1,
            "kind": "oracle",
            "sample": "whole tensor (%d bytes), %d compress+decompress round trips, best" % (n * w, reps)}


def run_offload_stream(args) -> int:
    """The VGG-16-style offload stream (16 ReLU outputs, batch 64): per-tensor codec
    rates, the aggregate, and the two-stream pipeline compress -> D2H -> H2D -> decompress
    against the same copies done uncompressed (the offload the paper starts from)."""
    import torch
    from paper_1705_01626_amd import workloads, zvc

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    specs = workloads.vgg_offload_stream()
    xs = [workloads.vgg_layer(s, i, args.seed, dev) for i, s in enumerate(specs)]
    caps = [zvc.zvc_max_compressed_bytes(x.numel(), 4) for x in xs]
    stages = [torch.empty(max(c, 16), dtype=torch.uint8, device=dev) for c in caps]
    pinned = [torch.empty(max(c, 16), dtype=torch.uint8, pin_memory=True) for c in caps]
    plain = [torch.empty(x.numel(), dtype=torch.float32, pin_memory=True) for x in xs]
    outs = [torch.empty_like(x) for x in xs]
    h_bytes = torch.zeros(1, dtype=torch.int64, pin_memory=True)
    d_bytes = torch.zeros(1, dtype=torch.int64, device=dev)
    ws = zvc.new_workspace(max(x.numel() for x in xs), 4, dev)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()

    def offload_all():
        sizes = []
        for x, st, hp in zip(xs, stages, pinned):
            sizes.append(zvc.zvc_offload(x, st, hp, h_bytes, ws, compute, copy))
        copy.synchronize()
        return sizes

    def prefetch_all(sizes):
        for x, st, hp, o, nb in reversed(list(zip(xs, stages, pinned, outs, sizes))):
            zvc.zvc_prefetch(hp, nb, st, o, ws, copy, compute)
        compute.synchronize()

    def plain_round_trip():
        with torch.cuda.stream(copy):
            for x, hp in zip(xs, plain):
                hp.copy_(x.view(-1), non_blocking=True)
        copy.synchronize()
        t_mid = time.perf_counter()
        with torch.cuda.stream(copy):
            for o, hp in reversed(list(zip(outs, plain))):
                o.view(-1).copy_(hp, non_blocking=True)
        copy.synchronize()
        return t_mid

    sizes = offload_all()
    prefetch_all(sizes)
    plain_round_trip()
    reps = max(1, min(args.steps, 5))
    t_off = t_pre = t_pd2h = t_ph2d = 0.0
    for _ in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        sizes = offload_all()
        t1 = time.perf_counter()
        prefetch_all(sizes)
        t2 = time.perf_counter()
        t_mid = plain_round_trip()
        t3 = time.perf_counter()
        t_off += t1 - t0
        t_pre += t2 - t1
        t_pd2h += t_mid - t2
        t_ph2d += t3 - t_mid
    for x, o in zip(xs, outs):
        assert torch.equal(x, o), "offload round trip differs"
    t_off, t_pre, t_pd2h, t_ph2d = (t / reps for t in (t_off, t_pre, t_pd2h, t_ph2d))

    # codec alone, per tensor, HIP events on the current stream
    layers, tc_all, td_all = [], 0.0, 0.0
    for spec, x, st, o, nb in zip(specs, xs, stages, outs, sizes):
        k = max(5, args.steps)
        ms_c = event_timed(lambda: zvc.zvc_compress(x, st, d_bytes, ws), k, torch)
        ms_d = event_timed(lambda: zvc.zvc_decompress(st, nb, o, ws), k, torch)
        ub = x.numel() * 4
        layers.append({"layer": spec.name, "bytes": ub, "density": round(spec.density, 4),
                       "ratio": round(ub / nb, 3), "compress_ms": round(ms_c, 5),
                       "decompress_ms": round(ms_d, 5),
                       "compress_hbm_frac": round((ub + nb) / (ms_c * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                       "decompress_hbm_frac": round((ub + nb) / (ms_d * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)})
        tc_all += ms_c
        td_all += ms_d
    total_in = sum(x.numel() * 4 for x in xs)
    total_out = sum(sizes)
    # the paper's bandwidth model (section 6) fed with what was just measured: kernel
    # times per tensor, the pinned-copy rate of this machine, and a size read-back per tensor
    from paper_1705_01626_amd import cdma_model
    link_gbps = total_in / t_pd2h / 1e9
    model_layers = [{"bytes": l["bytes"], "compressed_bytes": nb, "compress_s": l["compress_ms"] * 1e-3}
                    for l, nb in zip(layers, sizes)]
    model = cdma_model.predict(model_layers, link_gbps, host_gap_s=20e-6)
    model_out = {"link_GBps": round(link_gbps, 2), "host_gap_us_per_tensor": 20,
                 "predicted_offload_ms": round(model["offload_s"] * 1e3, 3),
                 "predicted_speedup": round(model["speedup"], 3),
                 "link_bound_ms": round(model["link_bound_s"] * 1e3, 3),
                 "compute_stream_ms": round(model["compute_stream_s"] * 1e3, 3),
                 "max_COMP_BW_needed_GBps": round(model["max_comp_bw_needed_gbps"], 1),
                 "min_encoder_read_GBps": round(model["min_encoder_read_gbps"], 1),
                 "layers_that_starve_the_link": model["layers_that_starve_the_link"],
                 "avg_codec_hbm_GBps": round(model["avg_codec_hbm_gbps"], 1),
                 "measured_over_predicted": round(t_off / model["offload_s"], 3)}
    print(json.dumps({
        "metric": "ZVC offload stream (VGG-16-style, batch 64): pipeline and codec rates",
        "value": round(2.0 * total_in / ((tc_all + td_all) * 1e-3) / 1e9, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": reps, "warmup": 1, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "config": {"workload": "vgg_offload", "tensors": 16, "uncompressed_bytes": total_in,
                   "compressed_bytes": total_out, "stream_ratio": round(total_in / total_out, 4)},
        "codec_aggregate": {"compress_ms": round(tc_all, 4), "decompress_ms": round(td_all, 4),
                            "hbm_frac": round((total_in + total_out) * 2 / ((tc_all + td_all) * 1e-3)
                                              / 1e9 / HBM_PEAK_GBPS, 4)},
        "pipeline": {"offload_ms": round(t_off * 1e3, 3), "prefetch_ms": round(t_pre * 1e3, 3),
                     "uncompressed_d2h_ms": round(t_pd2h * 1e3, 3),
                     "uncompressed_h2d_ms": round(t_ph2d * 1e3, 3),
                     "offload_speedup": round(t_pd2h / t_off, 3),
                     "prefetch_speedup": round(t_ph2d / t_pre, 3),
                     "d2h_GBps_compressed_bytes": round(total_out / t_off / 1e9, 2),
                     "d2h_GBps_uncompressed_copy": round(total_in / t_pd2h / 1e9, 2)},
        "cdma_model": model_out,
        "layers": layers}))
    return 0


def load_traffic(workload: str, direction: str):
    """HBM bytes per launch of one direction ("compress" / "decompress") from the committed
    rocprofv3 FETCH_SIZE / WRITE_SIZE runs (profiles/hbm_traffic.json), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        table = json.load(f)
    entry = table.get(workload)
    return entry[direction]["total"] if entry else None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="conv1_style")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--relu", action="store_true",
                    help="time the fused ReLU + ZVC encoder on pre-activations of the workload "
                         "(zeros of the tensor replaced by negative values)")
    ap.add_argument("--windowed", action="store_true",
                    help="time the paper-order windowed stream (zvc_window_compress / "
                         "zvc_window_decompress of all windows) instead of the planar one")
    ap.add_argument("--warm", action="store_true",
                    help="reuse one set of buffers (tensors under 512 MB then stay in the 256 MB "
                         "Infinity Cache); by default the calls rotate over enough copies to exceed 512 MB")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-verify", action="store_true")
    ap.add_argument("--counter-pass", action="store_true",
                    help="for rocprofv3 --pmc runs: a few rounds of [plain device copy of the "
                         "tensor, zvc_compress, zvc_decompress] and nothing else")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the hot path is single-GPU; "
              "see DESIGN.md for how it would shard); --gpus %d is refused" % args.gpus,
              file=sys.stderr)
        return 2

    import torch
    from paper_1705_01626_amd import zvc

    zvc.load()  # fails loudly if the HIP library is not built
    if args.workload == "vgg_offload":
        return run_offload_stream(args)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    x, described = make_workload(args.workload, args.seed, dev)
    x_in = x
    if args.relu:
        from paper_1705_01626_amd import workloads
        x_in = workloads.pre_activation(x.float(), args.seed + 1).to(x.dtype)
        x = torch.relu(x_in)          # what the round trip must give back
        described += "; pre-activations (zeros replaced by negative draws), fused ReLU + ZVC encoder"
    if args.relu and args.windowed:
        raise SystemExit("bench.py: --relu and --windowed are separate modes")
    encode = zvc.zvc_relu_compress if args.relu else zvc.zvc_compress
    n, w = x.numel(), x.element_size()
    if args.windowed:
        windows = zvc.zvc_window_count(n, w)
        offsets = torch.zeros(windows + 1, dtype=torch.int64, device=dev)
        described += "; paper-order stream in 1 KB windows with an offset table"

        def encode(t, c, b, s):
            zvc.zvc_window_compress(t, c, offsets, b, s)
    ws = zvc.new_workspace(n, w, dev)
    comp = zvc.new_compressed_buffer(n, w, dev)
    d_bytes = torch.zeros(1, dtype=torch.int64, device=dev)
    out = torch.empty_like(x)

    encode(x_in, comp, d_bytes, ws)
    nbytes = int(d_bytes.item())
    groups = (n + 31) // 32
    nnz = (nbytes - 4 * groups) // w
    density = nnz / n

    # Cold inputs: rotate over copies of the buffers whose inputs add up to more than 512 MB,
    # twice the Infinity Cache, so that no call finds its data cached by the previous one.
    copies = 1 if args.warm else max(1, -(-(512 << 20) // max(n * w, 1)))
    copies = min(copies, 64)
    sets = [(x_in, comp, out, offsets if args.windowed else None)]
    for _ in range(copies - 1):
        c2 = torch.empty_like(comp)
        o2 = offsets.clone() if args.windowed else None
        xi = x_in.clone()
        if args.windowed:
            zvc.zvc_window_compress(xi, c2, o2, d_bytes, ws)
        else:
            encode(xi, c2, d_bytes, ws)
        sets.append((xi, c2, torch.empty_like(x), o2))
    torch.cuda.synchronize()
    turn = {"c": 0, "d": 0}

    def compress():
        xi, c, _, o = sets[turn["c"] % copies]
        turn["c"] += 1
        if args.windowed:
            zvc.zvc_window_compress(xi, c, o, d_bytes, ws)
        else:
            encode(xi, c, d_bytes, ws)

    def decompress():
        _, c, o_t, o = sets[turn["d"] % copies]
        turn["d"] += 1
        if args.windowed:
            zvc.zvc_window_decompress(c, nbytes, o, n, 0, windows, o_t)
        else:
            zvc.zvc_decompress(c, nbytes, o_t, ws)

    def step():
        compress()
        decompress()

    if args.counter_pass:
        # the plain copy (n*w bytes read, n*w bytes written) calibrates the counters
        for _ in range(max(1, args.steps)):
            out.copy_(x)
            compress()
            decompress()
        torch.cuda.synchronize()
        print(json.dumps({"counter_pass": True, "workload": args.workload,
                          "uncompressed_bytes": n * w, "compressed_bytes": nbytes}))
        return 0

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    # per-kernel durations with HIP events on the launch stream
    ms_c = event_timed(compress, args.steps, torch)
    ms_d = event_timed(decompress, args.steps, torch)
    torch.cuda.synchronize()

    if not args.no_verify:
        turn["c"] = turn["d"] = 0
        for _ in range(copies):      # every set once more, whatever the step count was
            step()
        torch.cuda.synchronize()
        for _, _, o_t, _ in sets:
            assert torch.equal(o_t.view(torch.uint8), x.view(torch.uint8)), "round trip differs"
        assert int(d_bytes.item()) == nbytes

    uncompressed = n * w
    algorithmic = uncompressed + nbytes  # compress: read n*w, write stream; decompress: the mirror
    # The roofline kernel is compress_kernel: the one kernel of a zvc_compress call (zero
    # test, masks, scan, compaction, size) and the longest kernel of the step in rocprofv3's
    # trace; its call time is the kernel plus one launch gap.  zvc_decompress is two kernels
    # (mask pre-pass + expand) and is reported beside it as a whole call.
    dominant, ms_dom = "zvc_compress", ms_c
    achieved = algorithmic / (ms_dom * 1e-3) / 1e9
    traffic = load_traffic(args.workload, dominant[len("zvc_"):])
    result = {
        "metric": "ZVC compress+decompress GB/s (uncompressed bytes) and % of HBM peak",
        "value": round(2.0 * uncompressed / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32" if w == 4 else "u16",
        "data": "synthetic",
        "config": {"workload": args.workload, "tensor": described, "elements": n,
                   "element_bytes": w, "uncompressed_bytes": uncompressed,
                   "compressed_bytes": nbytes, "density": round(density, 6),
                   "compression_ratio": round(uncompressed / nbytes, 4), "seed": args.seed,
                   "encoder": "relu+zvc" if args.relu else "zvc",
                   "stream": "windowed" if args.windowed else "planar",
                   "buffers": "%d rotating set%s (%s)" % (copies, "" if copies == 1 else "s",
                                                           "warm" if args.warm else "cold inputs")},
        "compress_GBps": round(uncompressed / (ms_c * 1e-3) / 1e9, 2),
        "decompress_GBps": round(uncompressed / (ms_d * 1e-3) / 1e9, 2),
        "compress_ms": round(ms_c, 5),
        "decompress_ms": round(ms_d, 5),
        "hbm_peak_fraction": {"compress": round(algorithmic / (ms_c * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                              "decompress": round(algorithmic / (ms_d * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)},
        "roofline": {"bound": "hbm", "kernel": "compress_kernel", "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "algorithmic_bytes_per_launch": algorithmic,
                     "traffic": traffic},
    }
    if not args.no_cpu_baseline:
        host = x_in.view(torch.uint8).cpu().numpy().reshape(-1)
        result["cpu_baseline"] = cpu_baseline(host, n, w, relu=args.relu, windowed=args.windowed)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
