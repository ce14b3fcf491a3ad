#!/usr/bin/env python3
"""Benchmark of the Stripe block executor on one MI355X.

A step is one evaluation of one Stripe block (one stripe_block_run) on
synthetic seeded inputs that are resident in HBM before the timed region.
Default workload: the dense contraction block C[m,n] += A[m,k]*B[k,n],
M=N=K=4096, bf16 inputs, fp32 accumulate (the configuration the headline
metric is quoted on).  Other configurations can be timed with --workload;
the memory-bound ones rotate through several buffer sets so that the 256 MB
Infinity Cache cannot serve them.

Prints ONE JSON line with the throughput, the roofline record of the kernel
(measured live with HIP events on the launch stream) and the CPU oracle timed
on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"bf16_mfma_tflops": 2500.0, "int8_mfma_tops": 5000.0, "hbm_gbs": 8000.0, "fp32_vector_tflops": 157.3}

# Memory traffic per launch (bytes): FETCH_SIZE + WRITE_SIZE from the two rocprofv3 --pmc runs summarised under
# profiles/<workload>.md, each scaled by what the same counter reads for the 64 MiB copy kernel (x2.0 and x1.0).
# They are properties of the default kernel variants; --traffic-bytes overrides them after a fresh profile.
MEASURED_TRAFFIC = {
    "gemm_bf16_4096": 201.6e6 + 67.1e6,
    "resnet_conv_bf16": 16.9e6 + 25.7e6,
    "conv7x7_s2_int8": 3.4e6 + 51.4e6,
    "maxpool_f32": 120.2e6 + 25.7e6,
}
TRAFFIC_SOURCE = {name: f"profiles/{name}.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of the default kernel, scaled by profiles/device_copy.md)"
                  for name in MEASURED_TRAFFIC}

# workload -> (metric unit, bound, arithmetic dtype)
KIND = {
    "gemm_bf16_4096": ("TFLOP/s", "mfma", "bf16"),
    "resnet_conv_bf16": ("TFLOP/s", "hbm", "bf16"),
    "conv7x7_s2_int8": ("TOP/s", "hbm", "int8"),
    "maxpool_f32": ("GB/s", "hbm", "f32"),
    "tiny_conv_f32": ("TFLOP/s", "hbm", "f32"),
    "device_copy": ("GB/s", "hbm", "u8"),     # the plain copy kernel: calibrates traffic counters and the HBM yardstick
    "mfma_probe": ("TFLOP/s", "mfma", "bf16"),   # the matrix instruction on register-resident operands: the sustained compute roof
    "mfma_probe_lds": ("TFLOP/s", "mfma", "bf16"),   # the same with the operand fragments fetched from LDS for every pass
    # streaming yardsticks sized like the max-pooling block (102.8 MB in, 25.7 MB out): read only, write only, 1 : 1, 4 : 1
    "stream_read": ("GB/s", "hbm", "f32"),
    "stream_write": ("GB/s", "hbm", "f32"),
    "stream_1r1w": ("GB/s", "hbm", "f32"),
    "stream_4r1w": ("GB/s", "hbm", "f32"),
    "library_gemm": ("TFLOP/s", "mfma", "bf16"),  # torch.mm (the vendor BLAS) on the GEMM workload's operands: a yardstick
    # further shapes the kernel families cover (workloads.extra_block)
    "gemm_bf16_4096_bt": ("TFLOP/s", "mfma", "bf16"),
    "gemm_bf16_4000_ragged": ("TFLOP/s", "mfma", "bf16"),
    "gemm_i8_4096_bt": ("TOP/s", "mfma", "int8"),
    "gemm_bf16_1024": ("TFLOP/s", "mfma", "bf16"),
    "gemm_bf16_2048": ("TFLOP/s", "mfma", "bf16"),
    "gemm_bf16_256x256x65536": ("TFLOP/s", "mfma", "bf16"),    # split reduction (STRIPE_TUNE=gemm_splitk=0 times it unsplit)
    "gemm_i8_256x256x65536_bt": ("TOP/s", "mfma", "int8"),
    "gemm_bf16_1024x1024x8192": ("TFLOP/s", "mfma", "bf16"),
    "linear_bias_relu_4096": ("TFLOP/s", "mfma", "bf16"),
    # convolution shapes beyond the two tuned ones: the general matrix-core convolution kernel (--path generic: the fallback it replaces)
    "conv3x3_bf16_128to128": ("TFLOP/s", "mfma", "bf16"),
    "conv3x3_s2_bf16_64to128": ("TFLOP/s", "mfma", "bf16"),
    "conv1x7_bf16_64to64": ("TFLOP/s", "hbm", "bf16"),
    "conv3x3_bf16_w112": ("TFLOP/s", "hbm", "bf16"),
    "conv5x5_bf16_32to32": ("TFLOP/s", "hbm", "bf16"),
    "conv3x3_i8_64to64": ("TOP/s", "hbm", "int8"),
    "conv3x3_bf16_128to192": ("TFLOP/s", "mfma", "bf16"),
    "conv3x3_bf16_128to256_56": ("TFLOP/s", "mfma", "bf16"),
    "conv3x3_bf16_256to256_56": ("TFLOP/s", "mfma", "bf16"),
    "depthwise3x3_f32": ("GB/s", "hbm", "f32"),        # weighted windows on the pooling family's kernel
    "avgpool3x3s2_f32": ("GB/s", "hbm", "f32"),
    "maxpool2x2s2_f32": ("GB/s", "hbm", "f32"),
    "maxpool3x3s1_f32": ("GB/s", "hbm", "f32"),
    "pointwise_conv_bf16": ("TFLOP/s", "hbm", "bf16"),
    "transposed_conv_f32": ("TFLOP/s", "alu", "f32"),
    "resnet_conv_bias_relu_bf16": ("TFLOP/s", "hbm", "bf16"),   # two statements fused into one kernel, bf16 output
    "resnet_conv_bias_relu_f32": ("TFLOP/s", "hbm", "bf16"),
    "conv3x3_bias_relu_bf16_128to128": ("TFLOP/s", "mfma", "bf16"),   # the same fusion on the general convolution kernel
}


def oracle_sample(name, root, inputs, cores):
    """Time the oracle, as it stands, on a slab of the workload's outputs."""
    import numpy as np
    from oracle import stripe_oracle as O
    from paper_1903_06498_amd import workloads as W
    first = root.child
    lo, hi = [0] * len(first.ranges), list(first.ranges)
    if name == "gemm_bf16_4096":
        hi[0] = 32                       # 32 full output rows, every k: 537 M points (the whole block is 68.7 G points)
        sample, split = "32 of 4096 output rows (all n, all k), literal loops", 1
    elif name in ("resnet_conv_bf16", "conv7x7_s2_int8", "maxpool_f32"):
        sample, split = "the whole block (every image)", 0     # 3.6 G / 1.9 G / 57 M points: seconds on the host cores
    else:
        sample, split = "the whole block", 1
    np_ins = [W.to_numpy(t).ravel() for t in inputs]
    t0 = time.perf_counter()
    res = O.evaluate(root, np_ins, window=(lo, hi), threads=cores, split_index=split)
    dt = time.perf_counter() - t0
    return res, dt, sample, (lo, hi)


def bench_copy(args, torch, B):
    """stripe_device_copy of 64 MiB (128 MiB of traffic) over rotating buffer pairs."""
    dev = torch.device("cuda:0")
    n = 64 << 20
    pairs = [(torch.ones(n, dtype=torch.uint8, device=dev), torch.empty(n, dtype=torch.uint8, device=dev))
             for _ in range(args.rotate if args.rotate > 0 else 6)]
    stream = torch.cuda.current_stream()
    for i in range(args.warmup):
        s, d = pairs[i % len(pairs)]
        B.stripe_device_copy(s.data_ptr(), d.data_ptr(), n, stream.cuda_stream)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for i in range(args.steps):
        s, d = pairs[i % len(pairs)]
        B.stripe_device_copy(s.data_ptr(), d.data_ptr(), n, stream.cuda_stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    us = ev0.elapsed_time(ev1) / args.steps * 1e3
    gbs = 2 * n / us / 1e3
    print(json.dumps({"metric": "device copy bandwidth (yardstick)", "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us / 1e3, 5),
                      "higher_is_better": True, "dtype": "u8", "data": "synthetic",
                      "config": {"workload": "device_copy", "bytes_read": n, "bytes_written": n, "buffer_sets": len(pairs)},
                      "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK["hbm_gbs"], "unit": "GB/s",
                                   "frac": round(gbs / PEAK["hbm_gbs"], 4), "traffic": None, "kernel": "copy_kernel",
                                   "kernel_us": round(us, 2)}}), flush=True)


def bench_stream(args, torch, B, name):
    """stripe_device_stream with the pooling block's byte counts over rotating buffers; every grid size is timed and
    the best one is the yardstick (all of them are listed in config)."""
    dev = torch.device("cuda:0")
    n16 = 25690112 // 16                       # vectors per stream = the pooling block's output
    reads, write = {"stream_read": (4, 0), "stream_write": (0, 1), "stream_1r1w": (1, 1), "stream_4r1w": (4, 1)}[name]
    nbytes = 16 * n16 * (reads + write)
    n_sets = args.rotate if args.rotate > 0 else max(2, int(640e6 // nbytes) + 1)
    sets = [(torch.ones(max(1, reads) * n16 * 4, dtype=torch.float32, device=dev), torch.empty(n16 * 4, dtype=torch.float32, device=dev))
            for _ in range(n_sets)]
    stream = torch.cuda.current_stream()
    results = {}
    for grid in (512, 1024, 2048, 3136, 4096, 6272, 8192, 16384):
        run = lambda i: B.stripe_device_stream(sets[i % n_sets][0].data_ptr(), sets[i % n_sets][1].data_ptr(), n16, reads, write, grid,
                                               stream.cuda_stream)
        for i in range(args.warmup):
            run(i)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for i in range(args.steps):
            run(i)
        ev1.record(stream)
        torch.cuda.synchronize()
        results[grid] = ev0.elapsed_time(ev1) / args.steps * 1e3
    grid = min(results, key=results.get)
    us = results[grid]
    gbs = nbytes / us / 1e3
    print(json.dumps({"metric": "streaming bandwidth (yardstick)", "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us / 1e3, 5), "higher_is_better": True,
                      "dtype": "f32", "data": "synthetic",
                      "config": {"workload": name, "bytes_read": 16 * n16 * reads, "bytes_written": 16 * n16 * write, "buffer_sets": n_sets,
                                 "best_grid": grid, "us_by_grid": {str(k): round(v, 2) for k, v in results.items()}},
                      "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK["hbm_gbs"], "unit": "GB/s",
                                   "frac": round(gbs / PEAK["hbm_gbs"], 4), "traffic": None, "kernel": "stream_kernel", "kernel_us": round(us, 2)}}),
          flush=True)


def bench_mfma(args, torch, B, from_lds):
    """stripe_device_mfma: the contraction kernels' matrix instruction on operands resident in registers (mfma_probe) or
    fetched from LDS for every pass (mfma_probe_lds), one workgroup of four wavefronts per CU; operands N(0,1) rounded
    to bf16 (seed 0), or constant with --fill."""
    dev = torch.device("cuda:0")
    g = torch.Generator(device="cpu")
    g.manual_seed(0)
    ops = torch.randn((16 * 256, 8), generator=g, dtype=torch.float32).to(torch.bfloat16)
    ops = fill_like(ops, args.fill).to(dev)
    grid, iters = 256, 512
    out = torch.empty(grid * 256, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    run = lambda: B.stripe_device_mfma(ops.data_ptr(), out.data_ptr(), iters, grid, stream.cuda_stream, from_lds)
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(args.steps):
        run()
    ev1.record(stream)
    torch.cuda.synchronize()
    us = ev0.elapsed_time(ev1) / args.steps * 1e3
    flops = grid * 4 * iters * 16 * 32768.0
    tf = flops / us / 1e6
    print(json.dumps({"metric": "matrix-core rate on operands from " + ("LDS" if from_lds else "registers") + " (yardstick)", "value": round(tf, 2), "unit": "TFLOP/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us / 1e3, 5), "higher_is_better": True,
                      "dtype": "bf16", "data": "synthetic" if args.fill == "config" else f"diagnostic constant fill ({args.fill})",
                      "config": {"workload": "mfma_probe_lds" if from_lds else "mfma_probe", "grid": grid, "iters": iters, "instructions_per_wavefront": iters * 16, "fill": args.fill},
                      "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": PEAK["bf16_mfma_tflops"], "unit": "TFLOP/s",
                                   "frac": round(tf / PEAK["bf16_mfma_tflops"], 4), "traffic": None, "kernel": "mfma_probe_kernel",
                                   "kernel_us": round(us, 2), "algorithmic_flops": int(flops)}}), flush=True)


def sustained_mfma_roof(torch, B, dev, stream, warm=200, timed=100):
    g = torch.Generator(device="cpu")
    g.manual_seed(0)
    ops = torch.randn((16 * 256, 8), generator=g, dtype=torch.float32).to(torch.bfloat16).to(dev)
    grid, iters = 256, 512
    out = torch.empty(grid * 256, dtype=torch.float32, device=dev)
    run = lambda: B.stripe_device_mfma(ops.data_ptr(), out.data_ptr(), iters, grid, stream.cuda_stream, True)
    for _ in range(warm):
        run()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(timed):
        run()
    ev1.record(stream)
    torch.cuda.synchronize()
    us = ev0.elapsed_time(ev1) / timed * 1e3
    tf = grid * 4 * iters * 16 * 32768.0 / us / 1e6
    return {"value": round(tf, 1), "unit": "TFLOP/s", "kind": "32x32x16 bf16 matrix instructions on N(0,1) operands fetched from LDS, "
            "8 reads of 16 bytes per 16 instructions, no global traffic; %d launches after %d" % (timed, warm)}


def bench_library_gemm(args, torch, W):
    """The vendor library's bf16 x bf16 -> fp32 GEMM on the same seeded operands, same box, same clocks."""
    dev = torch.device("cuda:0")
    a, b = [t.to(dev) for t in W.config_inputs("gemm_bf16_4096")]
    a, b = fill_like(a, args.fill), fill_like(b, args.fill)
    f = lambda: torch.mm(a, b, out_dtype=torch.float32)
    for _ in range(args.warmup):
        f()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(args.steps):
        f()
    ev1.record()
    torch.cuda.synchronize()
    us = ev0.elapsed_time(ev1) / args.steps * 1e3
    tf = 2.0 * 4096 ** 3 / us / 1e6
    print(json.dumps({"metric": "vendor library GEMM (yardstick)", "value": round(tf, 2), "unit": "TFLOP/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us / 1e3, 5),
                      "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "library_gemm", "M": 4096, "N": 4096, "K": 4096, "fill": args.fill},
                      "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": PEAK["bf16_mfma_tflops"],
                                   "unit": "TFLOP/s", "frac": round(tf / PEAK["bf16_mfma_tflops"], 4), "traffic": None,
                                   "kernel": "torch.mm(out_dtype=float32)", "kernel_us": round(us, 2)}}), flush=True)


def fill_like(t, fill):
    """--fill diagnostic: operands of the same shape with all-equal values (low switching activity in the
    matrix cores).  The numbers of record use the seeded data ('config')."""
    if fill == "config":
        return t
    import torch
    return torch.zeros_like(t) if fill == "zeros" else torch.ones_like(t)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # 200 warm-up launches: under the 4096^3 GEMM the chip's power management needs on the order of 100 launches
    # (about 15 ms) to settle -- it first boosts, then over-corrects -- and the timed region should see the
    # sustained state (the per-launch series is in profiles/gemm_bf16_4096.md)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="gemm_bf16_4096", choices=sorted(KIND))
    ap.add_argument("--path", default="auto", help="force a kernel family (auto, generic, mfma_gemm, mfma_conv, pool)")
    ap.add_argument("--cpu-baseline", type=int, default=1, help="0 skips the oracle timing (profiling runs)")
    ap.add_argument("--rotate", type=int, default=-1, help="buffer sets to rotate through (-1: 1 for gemm, enough to exceed 512 MB otherwise)")
    ap.add_argument("--fill", default="config", choices=["config", "zeros", "ones"],
                    help="diagnostic: replace the seeded inputs by constants (shows how far the chip's power management, "
                         "not the kernel, sets the time); only 'config' is a valid measurement")
    ap.add_argument("--sustained-roof", type=int, default=1, help="default workload only.  1: before the warm-up, measure the matrix-core "
                    "rate the chip sustains (roofline.sustained_roof; 300 launches of the yardstick kernel, about 50 ms), so that the "
                    "yardstick and the timed steps see the same, settled power state; 2: the same after the timed region (a short "
                    "--warmup then starts from an idle chip, in the power management's transient); 0: skip")
    ap.add_argument("--traffic-bytes", type=float, default=None, help="HBM bytes per launch from rocprofv3 counters, if measured")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (every box here has one); --gpus must be 1")

    import torch
    from paper_1903_06498_amd import binding as B
    from paper_1903_06498_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP library has no CPU fallback")
    dev = torch.device("cuda:0")
    name = args.workload
    unit, bound, dtype = KIND[name]
    if name == "device_copy":
        return bench_copy(args, torch, B)
    if name == "library_gemm":
        return bench_library_gemm(args, torch, W)
    if name.startswith("stream_"):
        return bench_stream(args, torch, B, name)
    if name in ("mfma_probe", "mfma_probe_lds"):
        return bench_mfma(args, torch, B, name == "mfma_probe_lds")
    extra = name in W.EXTRA_NAMES
    root = W.extra_block(name) if extra else W.config_block(name)
    inputs = W.extra_inputs(name) if extra else W.config_inputs(name)
    if extra:
        args.cpu_baseline = 0        # the oracle is timed on the five configurations only
    blk = B.StripeBlock(root, args.path)
    info = blk.info
    ext = W.output_extent(root)
    odt = {"i32": torch.int32, "bf16": torch.bfloat16}.get(root.refs[-1].dtype, torch.float32)

    set_bytes = sum(t.numel() * t.element_size() for t in inputs) + ext * (2 if odt == torch.bfloat16 else 4)
    n_sets = args.rotate
    if n_sets < 1:
        n_sets = 1 if bound in ("mfma", "alu") else max(2, int(640e6 // set_bytes) + 1)
    sets = []
    for _ in range(n_sets):
        sets.append(([fill_like(t.to(dev), args.fill) for t in inputs], torch.zeros(ext, dtype=odt, device=dev)))
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    # raw device pointers, taken once: at 13 us per launch the binding's argument marshalling must not be what is timed
    ptr_sets = [([t.data_ptr() for t in ins], out.data_ptr()) for ins, out in sets]
    # The yardstick leg first: under the 4096^3 product the chip's power management boosts for about 14 launches from
    # idle, over-corrects for the next hundred and only then settles; 300 launches of the yardstick take it through
    # that, so a short --warmup / --steps pair measures the product on a chip that is already under load.
    sustained = None
    roof_leg = name == "gemm_bf16_4096" and args.fill == "config" and args.sustained_roof
    if roof_leg and args.sustained_roof == 1:
        sustained = sustained_mfma_roof(torch, B, dev, stream)
    for i in range(args.warmup):
        ins, out = ptr_sets[i % n_sets]
        blk.run(ins, out, stream.cuda_stream)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for i in range(args.steps):
        ins, out = ptr_sets[i % n_sets]
        blk.run(ins, out, stream.cuda_stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = ev0.elapsed_time(ev1)
    ms_per_step = wall_ms / args.steps
    kernel_s = gpu_ms / args.steps * 1e-3      # average launch duration over the timed region (events on the launch stream)

    work = info["work_points"]
    traffic, traffic_source = args.traffic_bytes, ("--traffic-bytes" if args.traffic_bytes is not None else None)
    if traffic is None and args.path == "auto" and not os.environ.get("STRIPE_TUNE") and args.fill == "config":
        traffic, traffic_source = MEASURED_TRAFFIC.get(name), TRAFFIC_SOURCE.get(name)
    flops = 2.0 * work
    nbytes = float(info["algorithmic_bytes"])
    if unit == "GB/s":
        value = nbytes / (ms_per_step * 1e-3) / 1e9
    else:
        value = flops / (ms_per_step * 1e-3) / 1e12
    if bound in ("mfma", "alu"):
        peak = PEAK["fp32_vector_tflops"] if bound == "alu" else PEAK["int8_mfma_tops"] if dtype == "int8" else PEAK["bf16_mfma_tflops"]
        achieved = flops / kernel_s / 1e12
        roof = {"bound": bound, "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 4), "traffic": traffic}
    else:
        achieved = nbytes / kernel_s / 1e9
        roof = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK["hbm_gbs"], "unit": "GB/s",
                "frac": round(achieved / PEAK["hbm_gbs"], 4), "traffic": traffic}
    if name == "tiny_conv_f32":
        # sub-microsecond of work: bound by launch latency, so the figure of merit is time per launch, not a roofline fraction
        roof = {"bound": "launch", "achieved": round(kernel_s * 1e6, 2), "peak": None, "unit": "us/launch", "frac": None, "traffic": None}
    if roof_leg:
        # the same kernel over 300 more launches directly after the timed region: the steady state, whatever --steps was
        ev2, ev3 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev2.record(stream)
        for i in range(300):
            ins, out = ptr_sets[i % n_sets]
            blk.run(ins, out, stream.cuda_stream)
        ev3.record(stream)
        torch.cuda.synchronize()
        steady_s = ev2.elapsed_time(ev3) / 300 * 1e-3
        roof["steady_state"] = {"kernel_us": round(steady_s * 1e6, 2), "achieved": round(flops / steady_s / 1e12, 2),
                                "frac": round(flops / steady_s / 1e12 / peak, 4), "launches": "300 directly after the timed region"}
        # what the chip sustains for this kernel's matrix instruction with operands of the same distribution fetched from
        # LDS at this kernel's ratio and nothing else going on (stripe_device_mfma)
        roof["sustained_roof"] = sustained if sustained is not None else sustained_mfma_roof(torch, B, dev, stream)
        roof["sustained_roof"]["measured"] = "before the warm-up" if sustained is not None else "after the timed region"
        roof["sustained_roof"]["frac_of_it"] = round(achieved / roof["sustained_roof"]["value"], 4)
    roof["traffic_source"] = traffic_source
    roof["kernel"] = info["kernel"]
    roof["kernel_us"] = round(kernel_s * 1e6, 2)
    roof["algorithmic_bytes"] = info["algorithmic_bytes"]
    roof["algorithmic_flops"] = int(flops)

    cpu = None
    if args.cpu_baseline and args.fill == "config":
        cores = min(16, os.cpu_count() or 1)
        res, dt, sample, _ = oracle_sample(name, root, inputs, cores)
        if unit == "GB/s":
            frac = res.n_points / max(1, work)
            cpu_value = nbytes * frac / dt / 1e9
        else:
            cpu_value = 2.0 * res.n_points / dt / 1e12
        cpu = {"value": float(f"{cpu_value:.6g}"), "unit": unit, "cores": cores, "kind": "oracle",
               "sample": f"{sample}: {res.n_points} points in {dt:.2f} s"}
        if name == "tiny_conv_f32":      # also on one core: the block is too small for threads to pay
            _, dt1, _, _ = oracle_sample(name, root, inputs, 1)
            cpu["single_thread_value"] = float(f"{2.0 * res.n_points / dt1 / 1e12:.6g}")
            cpu["sample"] += f"; one thread: {dt1 * 1e3:.2f} ms"

    line = {
        "metric": "Stripe block throughput: TFLOP/s (% of MFMA peak) for conv/matmul blocks, GB/s for max blocks",
        "value": round(value, 2), "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic" if args.fill == "config" else f"diagnostic constant fill ({args.fill})",
        "config": {"workload": name, "path": info["path_name"], "kernel": info["kernel"],
                   "tile": [info["tile_m"], info["tile_n"], info["tile_k"]], "grid": info["grid"],
                   "buffer_sets": n_sets, "hull_points": info["hull_points"], "work_points": work},
        "roofline": roof, "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)
    blk.close()


if __name__ == "__main__":
    main()
