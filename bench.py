#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

A "step" is one pass of every hot-path operation over one synthetic workload that is already resident
in HBM: compress(A), decompress, negate, multiply by a scalar, add(A, B), mean, dot, L2 norm, cosine
similarity, covariance, variance (B is compressed once, outside the timed region).

With no `--config` the run covers both 1 GiB workloads: the 512^3 FP64 volume in 4x4x4 blocks with int16
indices (the headline: `value`, `ms_per_step`, `ops`, `roofline`, `cpu_baseline` at the top level of the
JSON line are its figures) and the 1024x1024x512 bfloat16 volume in 8x8x8 blocks with int8 indices and
the 4x4x4 low-frequency box kept; each is timed for `--steps` steps after `--warmup` untimed ones, and
`workloads` holds the full record of both.  `--config N` times workload N alone (1..3: the smaller ones,
6: an MRI-like FP32 stack in 4x16x16 blocks, not one of the benchmark's five).

Per operation: time (HIP events on the launch stream, inside the timed region), GB/s of uncompressed input
(codec) or of compressed bytes read (reductions), GB/s of algorithmic bytes moved and that as a fraction of
the 8 TB/s HBM peak.  `roofline` describes the dominant kernel of the step, by measured time, and lists
both codec kernels; `cpu_baseline` is the FP64 numpy oracle timed on a bounded sample of the same workload
on this machine's host cores.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
LLC_BYTES = 256 * 1024 * 1024

# HBM bytes per launch of the two codec kernels from hardware counters: rocprofv3 --pmc FETCH_SIZE and --pmc
# WRITE_SIZE (KiB per dispatch), each scaled by what the same counter reads for pbz_stream_copy over the same
# 1 GiB array.  {workload: (profiles/ file the figures are taken from, {op: (KiB read, KiB written)})}
MEASURED_TRAFFIC_KIB = {
    "cfg2_2d_f32_b8x8_i16_mask4x4": ("profiles/hot_path_step__cfg2_4096sq_f32_8x8_i16_box4.md",
                                     {"compress": (65636.9, 9218.5), "decompress": (9324.1, 65578.0)}),
    "cfg3_series_f32_b1x16x16_i8": ("profiles/hot_path_step__cfg3_64x1024x1024_f32_1x16x16_i8.md",
                                    {"compress": (262309.7, 66564.4), "decompress": (66729.2, 262521.2)}),
    "cfg4_3d_f64_b4x4x4_i16": ("profiles/hot_path_step__cfg4_512cube_f64_4x4x4_i16.md",
                               {"compress": (1048708.7, 278528.0), "decompress": (278686.1, 1049358.8)}),
    "cfg5_3d_bf16_b8x8x8_i8_mask4x4x4": ("profiles/hot_path_step__cfg5_1024x1024x512_bf16_8x8x8_i8_box4.md",
                                         {"compress": (1048690.4, 69632.6), "decompress": (69722.1, 1049201.1)}),
}

# corner sub-array of A and B the oracle is timed on: roughly 10-30 s of host time per workload
CPU_SAMPLE = {1: (256, 256), 2: (4096, 4096), 3: (64, 1024, 1024), 4: (512, 512, 512), 5: (512, 1024, 512),
              6: (128, 512, 512)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=None, choices=[1, 2, 3, 4, 5, 6],
                    help="time this workload alone (default: the two 1 GiB workloads, 4 then 5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the operations timed outside the step (used for profiles of the step itself)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time replays of it (the per-operation times still "
                         "come from an eager pass with events); what a launch-bound caller of the small workloads does")
    ap.add_argument("--transform", default="dct", choices=["dct", "haar"],
                    help="orthonormal transform of the codec (the metric is quoted with the default, the DCT)")
    return ap.parse_args()


def cpu_baseline(wl, sample_shape, transform="dct"):
    """Time the oracle (as it stands) on a corner sub-array of A and B: the same step as the GPU's."""
    from oracle import pbz_oracle as po
    import threadpoolctl

    sl = tuple(slice(0, s) for s in sample_shape)
    a = wl.as_f64(np.ascontiguousarray(wl.A[sl]))
    b = wl.as_f64(np.ascontiguousarray(wl.B[sl]))
    cores = os.cpu_count() or 1
    try:
        cores = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        pass
    po.compress(a[tuple(slice(0, 2 * i) for i in wl.block)], wl.block, wl.index_bits, wl.ftype, wl.mask, transform)  # warm-up
    B = po.compress(b, wl.block, wl.index_bits, wl.ftype, wl.mask, transform)
    t0 = time.perf_counter()
    A = po.compress(a, wl.block, wl.index_bits, wl.ftype, wl.mask, transform)
    t_compress = time.perf_counter() - t0
    po.decompress(A)
    po.negate(A)
    po.multiply_scalar(A, -2.5)
    po.add(A, B)
    po.dot(A, B)
    po.norm2(A)
    has_dc = bool(A.P.reshape(-1)[0])
    if has_dc:
        po.mean(A)
        po.covariance(A, B)
        po.variance(A)
    po.cosine_similarity(A, B)
    dt = time.perf_counter() - t0
    in_bytes = a.size * wl.elem_bytes
    # the same compress with the numerical libraries held to one thread, on an eighth of the sample
    sl8 = tuple(slice(0, max(int(b), s // 2)) for s, b in zip(a.shape, wl.block)) if a.ndim == 3 else \
        tuple(slice(0, max(int(b), s // 3)) for s, b in zip(a.shape, wl.block))
    a8 = np.ascontiguousarray(a[sl8])
    with threadpoolctl.threadpool_limits(limits=1):
        t0 = time.perf_counter()
        po.compress(a8, wl.block, wl.index_bits, wl.ftype, wl.mask, transform)
        t_single = time.perf_counter() - t0
    return {"value": in_bytes / dt / 1e9, "unit": "GB/s of uncompressed input through one whole step",
            "cores": int(cores), "kind": "oracle",
            "sample": "corner sub-array %s of the workload's A and B (%d elements), one step, %.1f s; "
                      "compress alone %.3f GB/s; compress with the libraries on one thread %.3f GB/s"
                      % ("x".join(map(str, sample_shape)), a.size, dt, in_bytes / t_compress / 1e9,
                         a8.size * wl.elem_bytes / t_single / 1e9)}


def stream_copy_gbps(torch, api, x, y, repeats=5):
    """Rate of the library's plain copy kernel over the workload's uncompressed array (bytes read + written)."""
    api.stream_copy(y, x)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(repeats):
        api.stream_copy(y, x)
    c1.record()
    torch.cuda.synchronize()
    return 2 * x.numel() * x.element_size() * repeats / c0.elapsed_time(c1) / 1e6


def run_workload(config, args, torch, dev):
    """Times workload `config`; returns its record (the fields a single-workload JSON line is made of)."""
    from paper_2406_11209_amd import api, synth
    from paper_2406_11209_amd.api import Codec

    t_gen = time.perf_counter()
    wl = synth.make_workload(config)
    t_gen = time.perf_counter() - t_gen

    def up(x):
        if wl.dtype == "bf16":
            return torch.from_numpy(x.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(x).to(dev)

    xA, xB = up(wl.A), up(wl.B)
    codec = Codec(wl.block, wl.ftype, wl.index_bits, wl.mask, args.transform)
    lay = codec.layout(wl.shape)
    in_bytes = xA.numel() * xA.element_size()
    comp_bytes = lay.n_bytes + lay.f_bytes

    N1, F1 = codec.empty_compressed(wl.shape, dev)
    N2, F2 = codec.compress(xB)
    Nn, Fn = codec.empty_compressed(wl.shape, dev)   # outputs of the element-wise ops
    y = torch.empty_like(xA)
    scal = torch.empty(8, dtype=torch.float64, device=dev)
    has_dc = wl.mask is None or bool(np.asarray(wl.mask).reshape(-1)[0])

    # Cold caches for the small workloads: a step over less than about 600 MB would find its arrays in the
    # 256 MB last-level cache on the next step, so such workloads rotate through enough copies of every buffer
    # (inputs, compressed operands, outputs) that more than that is touched between two uses of one copy.
    step_bytes = 2 * in_bytes + 4 * comp_bytes
    n_sets = min(64, max(1, -(-600_000_000 // step_bytes)))
    sets = [(xA, N1, F1, N2, F2, Nn, Fn, y)]
    for _ in range(n_sets - 1):
        sets.append((xA.clone(), torch.empty_like(N1), torch.empty_like(F1), N2.clone(), F2.clone(),
                     torch.empty_like(Nn), torch.empty_like(Fn), torch.empty_like(y)))
    between_steps = "cold" if n_sets * step_bytes >= 600_000_000 else \
        "warm (the workload is too small to rotate out of the last-level cache)"
    rotation = [0]

    def rotate():
        nonlocal xA, N1, F1, N2, F2, Nn, Fn, y
        rotation[0] = (rotation[0] + 1) % n_sets
        xA, N1, F1, N2, F2, Nn, Fn, y = sets[rotation[0]]

    # (name, callable, algorithmic bytes moved, bytes the headline GB/s is quoted on).  Order: the codec, the
    # operations that write arrays, then the reductions.  Whatever follows a writer also waits for the tail of its
    # write-back (measured: the reduction placed right after `add` takes 20 us longer on the FP64 volume, whichever
    # reduction it is), so the light `mean` goes first among the reductions.
    ops = [
        ("compress", lambda: codec.compress(xA, N1, F1), in_bytes + comp_bytes, in_bytes),
        ("decompress", lambda: codec.decompress(N1, F1, wl.shape, out=y), in_bytes + comp_bytes, in_bytes),
        ("negate", lambda: codec.negate(F1, out=Fn), 2 * lay.f_bytes, lay.f_bytes),
        ("mul_scalar", lambda: codec.mul_scalar(N1, F1, -2.5, N_out=Nn, F_out=Fn), 2 * comp_bytes, comp_bytes),
        ("add", lambda: codec.add(N1, F1, N2, F2, N_out=Nn, F_out=Fn), 3 * comp_bytes, 2 * comp_bytes),
    ]
    if has_dc:
        dc_bytes = lay.n_bytes + lay.n_blocks * (lay.f_bytes // (lay.n_blocks * lay.kept_per_block))
        ops.append(("mean", lambda: codec.mean(N1, F1, out=scal[3:4]), dc_bytes, dc_bytes))
    ops += [
        ("dot", lambda: codec.dot(N1, F1, N2, F2, out=scal[0:1]), 2 * comp_bytes, 2 * comp_bytes),
        ("norm2", lambda: codec.norm2(N1, F1, out=scal[1:2]), comp_bytes, comp_bytes),
        ("cosine_similarity", lambda: codec.cosine_similarity(N1, F1, N2, F2, out=scal[2:3]), 2 * comp_bytes,
         2 * comp_bytes),
    ]
    if has_dc:
        ops += [
            ("covariance", lambda: codec.covariance(N1, F1, N2, F2, out=scal[4:5]), 2 * comp_bytes, 2 * comp_bytes),
            ("variance", lambda: codec.variance(N1, F1, out=scal[5:6]), comp_bytes, comp_bytes),
        ]
    reads_compressed_only = {"negate", "mul_scalar", "add", "mean", "dot", "norm2", "cosine_similarity", "covariance",
                             "variance"}

    def step(events=None):
        if n_sets > 1:
            rotate()
        for i, (_, fn, _, _) in enumerate(ops):
            if events is not None:
                events[i][0].record()
            fn()
            if events is not None:
                events[i][1].record()

    # The library's plain copy kernel over the uncompressed array: the box's practical streaming bandwidth, put
    # next to the 8 TB/s datasheet peak, and the reference dispatch that hardware-counter runs of this script
    # scale FETCH_SIZE / WRITE_SIZE by.
    copy_gbps = stream_copy_gbps(torch, api, xA, y)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in ops]
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(ev[k])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    steps = args.steps
    ms_per_step = dt / steps * 1e3
    if args.graph:
        # the same step recorded once (every call is a plain kernel launch on the current stream) and replayed
        # (one step per buffer set, so that a replay rotates through the sets like the eager loop does)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(n_sets):
                step()
        graph.replay()
        torch.cuda.synchronize()
        replays = max(1, args.steps // n_sets)
        t0 = time.perf_counter()
        for k in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        steps = replays * n_sets
        ms_per_step = (time.perf_counter() - t0) / steps * 1e3

    per_op = {}
    for i, (name, _, moved, quoted) in enumerate(ops):
        times = [ev[k][i][0].elapsed_time(ev[k][i][1]) for k in range(len(ev))]
        ms = float(np.mean(times))
        per_op[name] = {"ms": round(ms, 4), "ms_median": round(float(np.median(times)), 4),
                        "ms_min": round(float(np.min(times)), 4), "gbps": round(quoted / ms / 1e6, 1),
                        "gbps_moved": round(moved / ms / 1e6, 1),
                        "hbm_frac": round(moved / ms / 1e6 / HBM_PEAK_GBPS, 4)}
        # what the operation's operands can have found in the 256 MB last-level cache: within a step every
        # operation re-reads compressed arrays that the one before it wrote or read
        if name in reads_compressed_only and comp_bytes < LLC_BYTES:
            per_op[name]["operands"] = "in-step: a compressed operand fits the last-level cache, so hbm_frac is not pure HBM traffic"
        elif name in reads_compressed_only:
            per_op[name]["operands"] = "in-step: a compressed operand exceeds the last-level cache"
        else:
            per_op[name]["operands"] = "uncompressed array streamed from / to HBM"

    # operations beyond the base hot path, timed on their own after the timed region, not part of `value`
    extra_ops = {}
    Fm = torch.empty_like(F1)

    def difference_by_rebinning():        # the three-call route: negate, add (second binning), norm2
        codec.negate(F2, out=Fm)
        codec.add(N1, F1, N2, Fm, N_out=Nn, F_out=Fn)
        codec.norm2(Nn, Fn, out=scal[7:8])

    extras = [
        ("difference_norm2", lambda: codec.difference_norm2(N1, F1, N2, F2, out=scal[7:8]), 2 * comp_bytes),
        ("subtract", lambda: codec.subtract(N1, F1, N2, F2, N_out=Nn, F_out=Fn), 3 * comp_bytes),
        ("difference_norm2_via_negate_add_norm2", difference_by_rebinning, 2 * lay.f_bytes + 3 * comp_bytes + comp_bytes),
    ]
    if has_dc:
        # Algorithm 13: reads the first index and N of every block, then sorts two FP64 sequences of n_blocks
        extras.append(("approximate_wasserstein_p68",
                       lambda: codec.approximate_wasserstein(N1, F1, N2, F2, 68.0, out=scal[7:8]),
                       2 * (lay.n_bytes + lay.n_blocks * (lay.f_bytes // (lay.n_blocks * lay.kept_per_block)))))
        bw = torch.empty(lay.n_blocks, dtype=torch.float64, device=dev)
        bw_bytes = lay.n_blocks * 8
        st3 = torch.empty(3, dtype=torch.float64, device=dev)
        pair9 = torch.empty(9, dtype=torch.float64, device=dev)

        def compress_then_three_reductions():
            codec.compress(xA, N1, F1)
            codec.mean(N1, F1, out=st3[0:1])
            codec.variance(N1, F1, out=st3[1:2])
            codec.norm2(N1, F1, out=st3[2:3])

        def compress_then_one_pass():
            codec.compress(xA, N1, F1)
            codec.statistics(N1, F1, out=st3)

        extras += [
            # a time step compressed and its mean / variance / norm taken: fused, against the separate calls
            ("compress_statistics_fused", lambda: codec.compress_statistics(xA, N1, F1, out=st3), in_bytes + comp_bytes),
            ("compress_then_statistics_one_pass", compress_then_one_pass, in_bytes + 2 * comp_bytes),
            ("compress_then_mean_variance_norm2", compress_then_three_reductions, in_bytes + 3 * comp_bytes + dc_bytes),
            ("add_scalar", lambda: codec.add_scalar(N1, F1, 0.75, N_out=Nn, F_out=Fn), 2 * comp_bytes),
            ("ssim", lambda: codec.ssim(N1, F1, N2, F2, out=scal[6:7]), 2 * comp_bytes),
            # dot, cosine, covariance and both operands' mean / variance / norm from one pass over both
            ("pair_statistics_nine_values", lambda: codec.pair_statistics(N1, F1, N2, F2, out=pair9), 2 * comp_bytes),
            ("blockwise_mean", lambda: codec.blockwise_mean(N1, F1, out=bw), dc_bytes + bw_bytes),
            ("blockwise_variance", lambda: codec.blockwise_variance(N1, F1, out=bw), comp_bytes + bw_bytes),
            ("blockwise_covariance", lambda: codec.blockwise_covariance(N1, F1, N2, F2, out=bw), 2 * comp_bytes + bw_bytes),
        ]
        if wl.block[0] == 1 and len(wl.shape) == 3:
            # a time series: per-step statistics, all steps in one segmented call vs one call per step
            T = wl.shape[0]
            per = lay.n_blocks // T
            seg = torch.empty(T, dtype=torch.float64, device=dev)

            def per_step_variance():
                for t in range(T):
                    codec.variance(N1[t * per:(t + 1) * per], F1[t * per:(t + 1) * per], out=seg[t:t + 1])

            st_rows = torch.empty((T, 3), dtype=torch.float64, device=dev)

            def compress_one_call_per_step():
                for t in range(T):
                    codec.compress(xA[t:t + 1], N1[t * per:(t + 1) * per], F1[t * per:(t + 1) * per])

            def series_compress_then_segmented():
                codec.compress(xA, N1, F1)
                for k, name in enumerate(("mean", "variance", "norm2")):
                    codec.segmented(name, T, per, N1, F1, out=seg)

            extras += [
                # every step compressed and its mean / variance / norm emitted: one fused call vs compress + 3 segmented
                ("series_compress_statistics_per_step_fused",
                 lambda: codec.compress_statistics(xA, N1, F1, out=st_rows, per_step=True), in_bytes + comp_bytes),
                ("series_compress_then_three_segmented", series_compress_then_segmented,
                 in_bytes + 3 * comp_bytes + dc_bytes),
                ("series_mean_segmented", lambda: codec.segmented("mean", T, per, N1, F1, out=seg), dc_bytes),
                ("series_variance_segmented", lambda: codec.segmented("variance", T, per, N1, F1, out=seg), comp_bytes),
                ("series_covariance_consecutive_segmented",
                 lambda: codec.segmented("covariance", T - 1, per, N1, F1, N1[per:], F1[per:], out=seg[:T - 1]),
                 2 * comp_bytes * (T - 1) // T),
                ("series_variance_one_call_per_step", per_step_variance, comp_bytes),
                ("series_compress_one_call_per_step", compress_one_call_per_step, in_bytes + comp_bytes),
            ]
    for name, fn, moved in ([] if args.no_extras else extras):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        extra_ops[name] = {"ms": round(ms, 4), "gbps_moved": round(moved / ms / 1e6, 1),
                           "hbm_frac": round(moved / ms / 1e6 / HBM_PEAK_GBPS, 4)}

    # the dominant kernel of the step by measured time: one of the two codec kernels (each is a single launch
    # whose event time is its duration); both are listed
    traffic_file, traffic = MEASURED_TRAFFIC_KIB.get(wl.name, (None, {}))
    codec_kernels = {}
    for name in ("compress", "decompress"):
        rec = per_op[name]
        kib = traffic.get(name) if args.transform == "dct" else None
        codec_kernels[name] = {"kernel": codec.kernel_name(name, wl.shape, wl.dtype), "ms": rec["ms"],
                               "achieved": rec["gbps_moved"], "frac": round(rec["gbps_moved"] / HBM_PEAK_GBPS, 4),
                               "traffic": None if kib is None else int(round((kib[0] + kib[1]) * 1024)),
                               "frac_of_measured_copy": round(rec["gbps_moved"] / copy_gbps, 4)}
    dominant = max(codec_kernels, key=lambda n: codec_kernels[n]["ms"])
    dom = codec_kernels[dominant]
    roofline = {"bound": "hbm", "kernel": dom["kernel"] + " (" + dominant + ")", "achieved": dom["achieved"],
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": dom["frac"], "traffic": dom["traffic"],
                "traffic_source": traffic_file if dom["traffic"] is not None else None,
                "algorithmic_bytes_per_launch": in_bytes + comp_bytes,
                "measured_streaming_copy_gbps": round(copy_gbps, 1),
                "streaming_copy_kernel": "pbz_stream_copy over the workload's uncompressed array",
                "frac_of_measured_copy": dom["frac_of_measured_copy"],
                "codec_kernels": codec_kernels}

    record = {
        "value": round(in_bytes / (ms_per_step * 1e-3) / 1e9, 2),
        "ms_per_step": round(ms_per_step, 4),
        "steps": steps,
        "dtype": {"f64": "f64", "f32": "f32", "bf16": "f32"}[wl.dtype] if wl.index_bits == 8 or wl.ftype == "f64" else "f64",
        "config": {"workload": wl.name, "shape": list(wl.shape), "block": list(wl.block), "array_dtype": wl.dtype,
                   "index_bits": wl.index_bits, "kept_per_block": lay.kept_per_block, "transform": args.transform,
                   "launch": "hip graph replay" if args.graph else "eager",
                   "caches": "between steps: " + between_steps + "; within a step every operation follows the previous "
                             "one directly (see ops[*].operands)",
                   "buffer_sets": n_sets, "uncompressed_bytes": in_bytes, "compressed_bytes": comp_bytes,
                   "input_generation_s": round(t_gen, 1)},
        "ops": per_op,
        "extra_ops": extra_ops,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        record["cpu_baseline"] = cpu_baseline(wl, CPU_SAMPLE[config], args.transform)
    del sets, xA, xB, N1, F1, N2, F2, Nn, Fn, y, Fm
    gc.collect()
    torch.cuda.empty_cache()
    return record


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (blocks are independent, so an array shards by slabs of "
              "blocks and a reduction needs one exchange of its five partial sums); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    configs = [args.config] if args.config is not None else [4, 5]
    records = [run_workload(c, args, torch, dev) for c in configs]
    head = records[0]
    out = {
        "metric": "compress/decompress GB/s + compressed dot/L2-norm GB/s; fraction of HBM peak",
        "value": head["value"],
        "unit": "GB/s of uncompressed input through one whole hot-path step",
        "n_gpus": 1, "steps": head["steps"], "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic",
        "config": head["config"],
        "ops": head["ops"],
        "extra_ops": head["extra_ops"],
        "roofline": head["roofline"],
        # the paper gives its timings as figures only (Sec. IV-E, Fig. 2: RTX 3090, FP64 / int8 / 8x8 blocks;
        # Fig. 3: RTX 2070 Super; Fig. 8: hardware not stated), so there is no number to divide by
        "paper_timings": "not reported numerically (figures only: Fig. 2 on an RTX 3090, Fig. 3 on an RTX 2070 Super, Fig. 8)",
    }
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    if len(records) > 1:
        # every workload of the run, the headline included, each timed for the same number of steps
        out["workloads"] = {r["config"]["workload"]: r for r in records}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
