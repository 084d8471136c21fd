#!/usr/bin/env python3
"""Benchmark: images/sec through one model partition's forward + backward on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input already resident in
HBM: clear the gradient buffer, forward of all micro-batches, backward of all micro-batches
(each micro-batch on its own HIP stream), and -- for the whole-model configuration -- the SGD step.

    python bench.py [--steps K] [--warmup W] [--config 3]

Prints ONE JSON line.  `roofline` describes the kernel that takes the largest share of the step
(per-launch duration measured with HIP events on the launching stream, at the workload's shape,
through the single-kernel entry points); `kernels` lists every kernel class of the step the same
way; `cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
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


def kernel_classes(spec):
    """The step's kernel launches per micro-batch, grouped by (kind, shape): {key: count}.
    Mirrors the library's schedule: per block bn-relu before every conv; conv fwd / dgrad / wgrad."""
    from collections import Counter
    c = Counter()
    b = spec.microbatch
    h, w = spec.in_h, spec.in_w
    for blk in spec.blocks:
        ho, wo = h // blk.stride, w // blk.stride
        if blk.kind == 0:
            convs = [(blk.c_in, blk.c_mid, 3, blk.stride, h, w), (blk.c_mid, blk.c_out, 3, 1, ho, wo)]
        else:
            convs = [(blk.c_in, blk.c_mid, 1, blk.stride, h, w), (blk.c_mid, blk.c_mid, 3, 1, ho, wo),
                     (blk.c_mid, blk.c_out, 1, 1, ho, wo)]
        if blk.has_proj:
            convs.append((blk.c_in, blk.c_out, 1, blk.stride, h, w))
        for i, (ci, co, R, st, hi, wi) in enumerate(convs):
            if i < (2 if blk.kind == 0 else 3):
                c[("bn", b * hi * wi, ci)] += 1
            c[("conv", b, hi, wi, ci, co, R, st)] += 1
        h, w = ho, wo
    return c


def time_launches(torch, fn, iters=50, reps=6):
    """Average GPU time (s) of one fn() call: `iters` calls are captured into a graph on a side stream
    (so no host launch cost is in the figure) and the replays are bracketed by HIP events recorded on
    that same stream."""
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        fn()
        st.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            for _ in range(iters):
                fn()
        g.replay()
        st.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(reps):
            g.replay()
        e1.record(st)
        st.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / (iters * reps)


def probe_kernels(torch, hpf, spec, m):
    """Per-launch time of every kernel class at the workload's shapes.  Returns a list of dicts with
    algorithmic flops / bytes per launch and launches per step."""
    import numpy as np
    ops = hpf.Ops(hpf.HPF_BF16)
    dev = torch.device("cuda:0")
    out = []
    s = 2  # bytes per element
    for key, cnt in sorted(kernel_classes(spec).items(), key=str):
        if key[0] == "bn":
            _, M, C = key
            x = torch.randn(M, C, device=dev).to(torch.bfloat16)
            da = torch.randn(M, C, device=dev).to(torch.bfloat16)
            g = torch.ones(C, device=dev)
            bt = torch.zeros(C, device=dev)
            a, stats = ops.bn_relu_forward(x, g, bt)
            dx = torch.empty_like(x)
            t_f = time_launches(torch, lambda: ops.bn_relu_forward(x, g, bt, out=a))
            t_b = time_launches(torch, lambda: ops.bn_relu_backward(x, da, g, bt, stats, out=dx))
            # one call = 1 fill + 2 kernels; bytes: fwd 3*s*M*C (stats read, apply read+write), bwd 5*s*M*C
            out.append(dict(kernel="bn_relu_fwd(stats+apply)", shape=[M, C], launches_per_step=cnt * m, sec=t_f,
                            bytes=3 * s * M * C, flops=0, bound="hbm"))
            out.append(dict(kernel="bn_relu_bwd(reduce+apply)", shape=[M, C], launches_per_step=cnt * m, sec=t_b,
                            bytes=5 * s * M * C, flops=0, bound="hbm"))
        else:
            _, b, h, w, ci, co, R, st = key
            x = torch.randn(b, h, w, ci, device=dev).to(torch.bfloat16)
            wt = (torch.randn(R, R, ci, co, device=dev) * (2.0 / (R * R * ci)) ** 0.5)
            y = ops.conv_forward(x, wt, st)
            dy = torch.randn_like(y.float()).to(torch.bfloat16)
            dx = ops.conv_dgrad(dy, wt, (h, w), st)
            dw = ops.conv_wgrad(x, dy, R, st)
            M, K, N = b * (h // st) * (w // st), R * R * ci, co
            flops = 2.0 * M * K * N
            byt = s * (b * h * w * ci + K * N + M * N)
            # repack=False: the packed weight copies of the calls above are reused, one kernel per call
            t_f = time_launches(torch, lambda: ops.conv_forward(x, wt, st, out=y, repack=False))
            t_d = time_launches(torch, lambda: ops.conv_dgrad(dy, wt, (h, w), st, out=dx, repack=False))
            t_w = time_launches(torch, lambda: ops.conv_wgrad(x, dy, R, st, out=dw))
            shape = [M, K, N]
            out.append(dict(kernel="conv_fwd", shape=shape, launches_per_step=cnt * m, sec=t_f, bytes=byt, flops=flops, bound="mfma"))
            out.append(dict(kernel="conv_dgrad", shape=shape, launches_per_step=cnt * m, sec=t_d, bytes=byt, flops=flops, bound="mfma"))
            out.append(dict(kernel="conv_wgrad", shape=shape, launches_per_step=cnt * m, sec=t_w,
                            bytes=s * (b * h * w * ci + M * N) + 8 * K * N, flops=flops, bound="mfma"))
    return out


def cpu_baseline(spec, inputs, max_microbatches=4):
    """The oracle (fp32 storage, double sums, OpenMP) on the first micro-batches of the same workload."""
    import numpy as np
    import oracle
    from paper_1911_05146_amd import workloads as W
    n = min(spec.num_microbatches, max_microbatches)
    sub = W.with_microbatching(spec, spec.microbatch, n, loss_divisor=spec.divisor)
    sub_inp = W.StepInputs(inputs.params, inputs.act_in[:n], inputs.labels[:n] if inputs.labels else None,
                           inputs.err_in[:n] if inputs.err_in else None)
    oracle.lib()
    t0 = time.perf_counter()
    oracle.run_step(sub, sub_inp, np.float32)
    dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": sub.batch / dt, "unit": "images/s", "cores": cores, "kind": "oracle",
            "sample": f"{n} of {spec.num_microbatches} micro-batches ({sub.batch} images) forward+backward, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="benchmark configuration 1..5 (default 3: ResNet-1001 partition)")
    ap.add_argument("--schedule", choices=["grouped", "streams", "single-stream"], default="grouped",
                    help="grouped: all micro-batches of the batch in one group call per direction (default); "
                         "streams: one call and one stream per micro-batch; single-stream: one call per micro-batch, one stream")
    ap.add_argument("--no-graphs", action="store_true", help="plain kernel launches instead of HIP graph replay")
    ap.add_argument("--no-probe", action="store_true", help="skip the per-kernel probes")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
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
    spec = W.config(args.config)
    inputs = W.make_inputs(spec)
    m = spec.num_microbatches
    sgd = (0.1, 0.9) if args.config == 4 else None

    part = hpf.Partition(spec, inputs.params, hpf.HPF_BF16)
    if args.no_graphs:
        part.set_graphs(False)
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

    if args.calib_copy_mb > 0:
        src = torch.ones(args.calib_copy_mb << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    gbuf = torch.empty(part.n_params, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    if sgd is None:
        drain()
    img_s = spec.batch * args.steps / elapsed

    result = {
        "metric": "images/sec through partition fwd+bwd at 1 MI355X",
        "value": img_s, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"config {args.config}: {spec.name}, {len(spec.blocks)} blocks, "
                               f"{m} micro-batches of {spec.microbatch} images"
                               + (", + SGD step" if sgd else ""),
                   "batch": spec.batch, "microbatch": spec.microbatch, "num_microbatches": m,
                   "schedule": args.schedule, "hip_graphs": not args.no_graphs},
    }

    if not args.no_probe:
        ks = probe_kernels(torch, hpf, spec, m)
        for k in ks:
            k["share_sec_per_step"] = k["sec"] * k["launches_per_step"]
        dom = max(ks, key=lambda k: k["share_sec_per_step"])
        if dom["bound"] == "mfma":
            ach, peak, unit = dom["flops"] / dom["sec"] / 1e12, PEAK_MFMA_BF16 / 1e12, "TFLOP/s"
        else:
            ach, peak, unit = dom["bytes"] / dom["sec"] / 1e9, PEAK_HBM / 1e9, "GB/s"
        result["roofline"] = {"bound": dom["bound"], "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
                              "traffic": None, "kernel": dom["kernel"], "shape": dom["shape"],
                              "avg_launch_us": dom["sec"] * 1e6,
                              "hbm_frac_of_same_kernel": dom["bytes"] / dom["sec"] / PEAK_HBM}
        result["kernels"] = [
            {"kernel": k["kernel"], "shape": k["shape"], "launches_per_step": k["launches_per_step"],
             "avg_us": round(k["sec"] * 1e6, 2),
             "TFLOP/s": round(k["flops"] / k["sec"] / 1e12, 2) if k["flops"] else None,
             "mfma_frac": round(k["flops"] / k["sec"] / PEAK_MFMA_BF16, 4) if k["flops"] else None,
             "GB/s": round(k["bytes"] / k["sec"] / 1e9, 1), "hbm_frac": round(k["bytes"] / k["sec"] / PEAK_HBM, 4)}
            for k in ks]
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(spec, inputs)
    part.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
