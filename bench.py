#!/usr/bin/env python3
"""Benchmark: images/sec through one model partition's forward + backward on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input already resident in
HBM: clear the gradient buffer, forward of all micro-batches, backward of all micro-batches
(each micro-batch on its own HIP stream), and -- for the whole-model configuration -- the SGD step.

    python bench.py [--steps K] [--warmup W] [--config 3]

Prints ONE JSON line.  `roofline` describes the kernel class that takes the largest share of the
step: its per-launch duration is measured with HIP events on the launching stream, in the launch
configuration that was timed, by the library's profiling mode (ten more steps after the timed
region); `kernels` lists every kernel class of the step the same way; `cpu_baseline` is the CPU
oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_BF16 = 2.5e15   # dense bf16 MFMA flop/s, MI355X
PEAK_HBM = 8.0e12         # bytes/s


# HBM bytes per launch from rocprofv3 counter runs of this same command (FETCH_SIZE + WRITE_SIZE, each
# scaled by what the counter reads for a plain device copy of known size); the summaries with the
# commands are under profiles/.  Keyed by (kernel class, configuration).
MEASURED_TRAFFIC = {("resident_backward", 3): 1.150e9}
TRAFFIC_SOURCE = ("constant taken from profiles/hbm_traffic_resnet1001_partition.md (two rocprofv3 --pmc runs of this "
                  "command), not measured in this run")


def profile_classes(torch, part, step, steps=10):
    """Per-kernel-class GPU time of the step in the launch configuration that was just timed: the library
    brackets every class with HIP events on the launching stream (plain launches instead of graph replay
    while it does).  Returns the library's entries with per-launch averages added."""
    part.set_profiling(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    entries = part.profile_read()
    part.set_profiling(False)
    for e in entries:
        e["avg_sec"] = e["total_ms"] * 1e-3 / e["launches"]
        e["launches_per_step"] = e["launches"] / steps
        e["sec_per_step"] = e["total_ms"] * 1e-3 / steps
    return entries


def measured_ceilings(torch, dev):
    """What this chip achieves on a plain copy and on a register-only MFMA loop (the library's two probe kernels),
    timed with events on the launch stream: the ceilings to read the kernel rates against next to the data-sheet ones."""
    from paper_1911_05146_amd import hpf
    stream = torch.cuda.current_stream(dev)
    nbytes = 1 << 30
    src = torch.ones(nbytes, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    wgs, iters = 4096, 2048
    sink = torch.empty(wgs * 256, dtype=torch.float32, device=dev)

    def timed(fn, reps):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    t_copy = timed(lambda: hpf.hpf_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream.cuda_stream), 10)
    flops = float(wgs) * 4 * iters * 131072
    t_mfma = {shape: timed(lambda: hpf.hpf_probe_mfma_bf16(sink.data_ptr(), wgs, iters, wide, stream.cuda_stream), 5)
              for shape, wide in (("16x16x32", False), ("32x32x16", True))}
    best = min(t_mfma, key=t_mfma.get)
    del src, dst, sink
    return {"copy_GB/s": 2 * nbytes / t_copy / 1e9, "copy": "1 GiB read + 1 GiB written per launch",
            "mfma_bf16_TFLOP/s": flops / t_mfma[best] / 1e12,
            "mfma": f"{wgs} work-groups x 4 waves x {iters} rounds of 131072 flop, v_mfma_f32_{best}_bf16 "
                    f"(16x16x32: {flops / t_mfma['16x16x32'] / 1e12:.0f}, 32x32x16: {flops / t_mfma['32x32x16'] / 1e12:.0f} TFLOP/s)"}


def cpu_baseline(spec, inputs, max_microbatches=None, threads=None, repeats=3):
    """The oracle as it stands (fp32 storage, double sums, OpenMP) on the same workload: the full step on all
    threads, best of `repeats`; or, with max_microbatches, on the first micro-batches only.
    threads: ask the OpenMP runtime for this many threads first (the oracle itself has no such setting)."""
    import numpy as np
    import oracle
    from paper_1911_05146_amd import workloads as W
    if threads is not None:
        import ctypes
        ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(threads))
    n = min(spec.num_microbatches, max_microbatches or spec.num_microbatches)
    sub = W.with_microbatching(spec, spec.microbatch, n, loss_divisor=spec.divisor)
    sub_inp = W.StepInputs(inputs.params, inputs.act_in[:n], inputs.labels[:n] if inputs.labels else None,
                           inputs.err_in[:n] if inputs.err_in else None)
    oracle.lib()
    times = []
    for _ in range(max(1, repeats)):
        t0 = time.perf_counter()
        oracle.run_step(sub, sub_inp, np.float32)
        times.append(time.perf_counter() - t0)
    dt = min(times)
    cores = int(threads) if threads is not None else int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    what = "the full step" if n == spec.num_microbatches else f"{n} of {spec.num_microbatches} micro-batches"
    return {"value": sub.batch / dt, "unit": "images/s", "cores": cores, "kind": "oracle",
            "sample": f"{what} ({sub.batch} images) forward+backward, best of {len(times)}: {dt:.1f} s"}


def bench_pipeline(args, torch, dev):
    """Whole ResNet-110 (54 basic blocks, 32x32x3 inputs, 8 micro-batches of 16) as P chained partitions."""
    from paper_1911_05146_amd import hpf, layer_cuts, workloads as W
    from paper_1911_05146_amd.pipeline import Pipeline, split_model
    blocks, b, m, seed = W.basic_resnet_blocks(18), 16, 8, W.SEED_BASE + 6
    if args.cuts == "layers":
        cm = layer_cuts.split_at_layers("resnet110", blocks, layer_cuts.even_layer_cuts(blocks, args.pipeline), 32, 16, 10, b, m, seed)
        specs, whole = cm.specs, cm.whole
    else:
        cm = None
        specs = split_model("resnet110", blocks, args.pipeline, 32, 16, 10, b, m, seed)
        whole = W.partition_of("resnet110", blocks, 1, 0, 32, 16, 16, 10, b, m, seed)
    inp = W.make_inputs(whole)
    pipe = Pipeline(specs, inp.params, hpf.HPF_BF16, group=1 if cm else args.group, cut_model=cm)
    x = [torch.from_numpy(a).to(dev) for a in inp.act_in]
    lab = [torch.from_numpy(l).to(dev) for l in inp.labels]

    def step():
        for part, s in zip(pipe.parts, pipe.streams):
            part.grad_accum_zero(stream=s)
        pipe.run_batch(x, lab)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    n_skip = sum(1 for msg in cm.messages if msg.tensor == "skip") if cm else 0
    pipe.close()
    print(json.dumps({
        "metric": "images/sec through the chained partitions fwd+bwd at 1 MI355X", "value": b * m * args.steps / elapsed,
        "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"ResNet-110 whole model, {args.pipeline} partitions cut at {args.cuts}, "
                               f"{m} micro-batches of {b} images, one stream per partition, "
                               f"{1 if cm else args.group} micro-batch(es) per call",
                   "partitions": args.pipeline, "cuts": args.cuts, "skip_tensors_crossing_partitions": n_skip}}))


def bench_bn(args, torch, dev):
    """The stand-alone BN+ReLU kernels on a [12544, C] bf16 tensor: algorithmic bytes per call over event time."""
    from paper_1911_05146_amd import hpf
    M, Cc = 12544, args.bn_bandwidth
    ops = hpf.Ops(hpf.HPF_BF16)
    g = torch.Generator(device="cpu").manual_seed(191105146)
    x = torch.randn((M, Cc), generator=g).to(dev, torch.bfloat16)
    da = torch.randn((M, Cc), generator=g).to(dev, torch.bfloat16)
    gamma = torch.ones(Cc, device=dev)
    beta = torch.zeros(Cc, device=dev)
    a, dx = torch.empty_like(x), torch.empty_like(x)
    stream = torch.cuda.current_stream(dev)
    if args.calib_copy_mb > 0:       # one plain copy of known size in the same process: the yardstick of the HBM counters
        src = torch.ones(args.calib_copy_mb << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        hpf.hpf_probe_copy(dst.data_ptr(), src.data_ptr(), src.numel(), stream.cuda_stream)
        torch.cuda.synchronize()

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            fn()
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / args.steps

    _, stats = ops.bn_relu_forward(x, gamma, beta, out=a)
    t_f = timed(lambda: ops.bn_relu_forward(x, gamma, beta, out=a))
    t_b = timed(lambda: ops.bn_relu_backward(x, da, gamma, beta, stats, out=dx))
    sMC = 2.0 * M * Cc
    print(json.dumps({"metric": "achieved HBM GB/s of the stand-alone BatchNorm+ReLU kernels at 1 MI355X", "unit": "GB/s",
                      "shape": [M, Cc], "dtype": "bf16", "steps": args.steps,
                      "forward": {"us": t_f * 1e6, "algorithmic_bytes": 3 * sMC, "GB/s": 3 * sMC / t_f / 1e9, "frac_of_8TB/s": 3 * sMC / t_f / PEAK_HBM,
                                  "kernels": "k_bn_stats (reads x) + k_bn_stats_finalize + k_bn_apply_relu (reads x, writes a)"},
                      "backward": {"us": t_b * 1e6, "algorithmic_bytes": 5 * sMC, "GB/s": 5 * sMC / t_b / 1e9, "frac_of_8TB/s": 5 * sMC / t_b / PEAK_HBM,
                                   "kernels": "k_bn_bwd_reduce (reads x, da) + k_bn_bwd_finalize + k_bn_bwd_apply (reads x, da, writes dx)"}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="benchmark configuration 1..8 (default 3: ResNet-1001 partition; 6: the same cut of the 30 M-parameter variant; 7: ResNet-110-v1 whole; 8: VGG-16 whole)")
    ap.add_argument("--schedule", choices=["grouped", "streams", "single-stream"], default="grouped",
                    help="grouped: all micro-batches of the batch in one group call per direction (default); "
                         "streams: one call and one stream per micro-batch; single-stream: one call per micro-batch, one stream")
    ap.add_argument("--no-graphs", action="store_true", help="plain kernel launches instead of HIP graph replay")
    ap.add_argument("--fusion", type=int, choices=[0, 1, 2], default=2,
                    help="kernel schedule of the library (hpf_partition_set_fusion); default 2, the library's default")
    ap.add_argument("--no-probe", action="store_true", help="skip the per-kernel-class timing")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--pipeline", type=int, default=0, metavar="P",
                    help="instead of one partition: the whole ResNet-110 (CIFAR shape) cut into P partitions chained on "
                         "the GPU, one stream per partition (paper: pipelined model parallelism); see --cuts")
    ap.add_argument("--group", type=int, default=1,
                    help="with --pipeline and --cuts blocks: micro-batches per library call (1, 2, 4 or 8)")
    ap.add_argument("--cuts", choices=["blocks", "layers"], default="blocks",
                    help="with --pipeline: cut at residual-block boundaries, or evenly over the convolution layers "
                         "(cuts inside blocks; shortcut values cross partitions)")
    ap.add_argument("--inference", action="store_true",
                    help="instead of training steps: inference forwards (BatchNorm by running statistics) of the "
                         "configuration's micro-batches, one call each")
    ap.add_argument("--no-cpu-one-core", action="store_true",
                    help="skip the oracle timing on one thread (one micro-batch; a few seconds)")
    ap.add_argument("--cpu-repeats", type=int, default=3, help="the all-thread oracle timing is the best of this many full steps")
    ap.add_argument("--no-others", dest="others", action="store_false",
                    help="skip the short runs of the other configurations that follow the headline one")
    ap.add_argument("--bn-bandwidth", type=int, default=0, metavar="C",
                    help="instead of a partition: the stand-alone BatchNorm+ReLU kernels (statistics, normalise+ReLU, backward "
                         "reduction, backward apply) on one [12544, C] bf16 tensor (the ResNet-152 stage-3 shape), --steps times; "
                         "prints achieved GB/s of the forward and the backward pair from HIP events (per-kernel times: run under "
                         "rocprofv3 --kernel-trace --stats)")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also run one plain device copy of this many MiB (reference for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one partition on ONE GPU; --gpus must be 1 "
              "(no collectives or multi-GPU sharding are part of it)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1911_05146_amd import hpf, workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.pipeline > 0:
        return bench_pipeline(args, torch, dev)
    if args.bn_bandwidth > 0:
        return bench_bn(args, torch, dev)
    result = run_config(args, torch, dev, args.config, args.steps, args.warmup, probe=not args.no_probe, cpu=not args.no_cpu)
    if result is None:
        return
    if args.others:
        # the other configurations, after the timed region of the headline one: shorter runs, same launch configuration
        result["other_configs"] = []
        for cfg in (1, 2, 4, 5, 6, 7, 8):
            if cfg == args.config:
                continue
            r = run_config(args, torch, dev, cfg, max(5, args.steps // 3), 3, probe=not args.no_probe, cpu=False, ceilings=False)
            entry = {"config": cfg, "workload": r["config"]["workload"], "ms_per_step": r["ms_per_step"], "images/s": r["value"],
                     "steps": r["steps"], "warmup": r["warmup"]}
            if "roofline" in r:
                rf = r["roofline"]
                entry["dominant_kernel_class"] = rf["kernel"]
                entry["roofline"] = {k: rf[k] for k in ("bound", "achieved", "peak", "unit", "frac", "avg_launch_us", "launches_per_step",
                                                        "share_of_step_gpu_time")}
                entry["kernels"] = r["kernels"]
            result["other_configs"].append(entry)
    print(json.dumps(result))


def run_config(args, torch, dev, config, steps, warmup, probe=True, cpu=True, ceilings=True):
    """Times `steps` steps of one configuration; returns the result dictionary (None: a mode that printed its own line)."""
    import numpy as np  # noqa: F401
    from paper_1911_05146_amd import hpf, workloads as W
    spec = W.config(config)
    inputs = W.make_inputs(spec)
    m = spec.num_microbatches
    sgd = (0.1, 0.9) if config in (4, 7, 8) else None   # the whole models take the SGD step too

    part = hpf.Partition(spec, inputs.params, hpf.HPF_BF16)
    if args.no_graphs:
        part.set_graphs(False)
    if args.fusion != 2:
        part.set_fusion(args.fusion)
    tdt = torch.bfloat16
    act_in = [torch.from_numpy(a).to(dev, torch.float32 if spec.has_stem else tdt) for a in inputs.act_in]
    labels = [torch.from_numpy(l).to(dev) for l in inputs.labels] if inputs.labels else [None] * m
    err_in = [torch.from_numpy(e).to(dev, tdt) for e in inputs.err_in] if inputs.err_in else [None] * m
    act_out = [None if spec.has_head else torch.empty(part.out_shape, dtype=tdt, device=dev) for _ in range(m)]
    err_out = [None if spec.has_stem else torch.empty(part.in_shape, dtype=tdt, device=dev) for _ in range(m)]
    main_stream = torch.cuda.Stream(dev)
    streams = [torch.cuda.Stream(dev) for _ in range(m)] if args.schedule == "streams" else [main_stream] * m
    lab_list = labels if inputs.labels else None
    out_list = None if spec.has_head else act_out
    ein_list = None if spec.has_head else err_in
    eout_list = None if spec.has_stem else err_out

    def step():
        if sgd is None:
            part.grad_accum_zero(stream=main_stream)
        if args.schedule == "grouped":
            part.forward_microbatches(0, act_in, lab_list, out_list, stream=main_stream)
            part.backward_microbatches(0, m, ein_list, eout_list, stream=main_stream)
        else:
            for i in range(m):
                part.forward_microbatch(i, act_in[i], labels[i], act_out[i], stream=streams[i])
            for i in range(m):
                part.backward_microbatch(i, err_in[i], err_out[i], stream=streams[i])
        if sgd is not None:
            part.sgd_step(*sgd, stream=main_stream)

    def drain():
        # the last step's backward work sits on the micro-batch streams: join them
        part.grad_accum_read(out=gbuf, stream=main_stream) if sgd is None else None
        torch.cuda.synchronize()

    if args.inference:
        xs = act_in
        skips = None
        oshape = (spec.microbatch, spec.num_classes) if spec.has_head else part.out_shape
        outs = [torch.empty(oshape, dtype=torch.float32 if spec.has_head else tdt, device=dev) for _ in xs]

        def infer_all():
            if args.schedule == "grouped":
                for i in range(0, len(xs), 8):
                    part.forward_inference_group(xs[i:i + 8], stream=main_stream, out=outs[i:i + 8])
            else:
                for x, o in zip(xs, outs):
                    part.forward_inference(x, stream=main_stream, out=o)

        for _ in range(warmup):
            infer_all()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            infer_all()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        part.close()
        print(json.dumps({
            "metric": "images/sec through partition inference forward at 1 MI355X", "value": spec.batch * steps / elapsed,
            "unit": "images/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": elapsed / steps * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"config {config}: {spec.name}, inference forward of {m} micro-batches of "
                                   f"{spec.microbatch} images, " + ("one group call" if args.schedule == "grouped" else "one call each")}}))
        return None

    if args.calib_copy_mb > 0:
        src = torch.ones(args.calib_copy_mb << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    gbuf = torch.empty(part.n_params, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    if sgd is None:
        drain()
    part.check()   # a resident launch that gave up waiting would have left invalid gradients: fail loudly
    img_s = spec.batch * steps / elapsed

    result = {
        "metric": "images/sec through partition fwd+bwd at 1 MI355X",
        "value": img_s, "unit": "images/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": elapsed / steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"config {config}: {spec.name}, {len(spec.blocks)} blocks, "
                               f"{m} micro-batches of {spec.microbatch} images"
                               + (", + SGD step" if sgd else ""),
                   "batch": spec.batch, "microbatch": spec.microbatch, "num_microbatches": m,
                   "schedule": args.schedule, "hip_graphs": not args.no_graphs, "fusion_level": args.fusion},
    }

    if probe:
        ks = profile_classes(torch, part, step)
        if sgd is None:
            drain()
        # the class with the largest share of the step's GPU time among those with algorithmic figures
        dom = max([k for k in ks if k["bytes_per_launch"] > 0 or k["flops_per_launch"] > 0] or ks, key=lambda k: k["sec_per_step"])
        gbs = dom["bytes_per_launch"] / dom["avg_sec"] / 1e9
        tfl = dom["flops_per_launch"] / dom["avg_sec"] / 1e12
        # the roof the kernel is closer to
        if dom["bytes_per_launch"] > 0 and gbs / (PEAK_HBM / 1e9) >= tfl / (PEAK_MFMA_BF16 / 1e12):
            bound, ach, peak, unit = "hbm", gbs, PEAK_HBM / 1e9, "GB/s"
        else:
            bound, ach, peak, unit = "mfma", tfl, PEAK_MFMA_BF16 / 1e12, "TFLOP/s"
        result["roofline"] = {"bound": bound, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
                              "traffic": MEASURED_TRAFFIC.get((dom["name"], config)),
                              "traffic_source": TRAFFIC_SOURCE if (dom["name"], config) in MEASURED_TRAFFIC else None,
                              "kernel": dom["name"],
                              "avg_launch_us": dom["avg_sec"] * 1e6, "launches_per_step": dom["launches_per_step"],
                              "algorithmic_bytes_per_launch": dom["bytes_per_launch"],
                              "algorithmic_flops_per_launch": dom["flops_per_launch"],
                              "share_of_step_gpu_time": dom["sec_per_step"] / sum(k["sec_per_step"] for k in ks)}
        result["kernels"] = [
            {"kernel": k["name"], "launches_per_step": k["launches_per_step"], "avg_us": round(k["avg_sec"] * 1e6, 2),
             "us_per_step": round(k["sec_per_step"] * 1e6, 1),
             "TFLOP/s": round(k["flops_per_launch"] / k["avg_sec"] / 1e12, 2) if k["flops_per_launch"] else None,
             "mfma_frac": round(k["flops_per_launch"] / k["avg_sec"] / PEAK_MFMA_BF16, 4) if k["flops_per_launch"] else None,
             "GB/s": round(k["bytes_per_launch"] / k["avg_sec"] / 1e9, 1) if k["bytes_per_launch"] else None,
             "hbm_frac": round(k["bytes_per_launch"] / k["avg_sec"] / PEAK_HBM, 4) if k["bytes_per_launch"] else None}
            for k in ks]
    if probe and ceilings:
        ceil = measured_ceilings(torch, dev)
        result["measured_ceilings"] = ceil
        r = result["roofline"]
        r["frac_of_measured_ceiling"] = r["achieved"] / (ceil["copy_GB/s"] if r["bound"] == "hbm" else ceil["mfma_bf16_TFLOP/s"])
    if cpu:
        result["cpu_baseline"] = cpu_baseline(spec, inputs, repeats=args.cpu_repeats)
        if not args.no_cpu_one_core:   # after the all-thread run: the thread count stays at 1 from here on
            result["cpu_baseline"]["one_core"] = cpu_baseline(spec, inputs, max_microbatches=1, threads=1, repeats=1)
    part.close()
    return result


if __name__ == "__main__":
    main()
