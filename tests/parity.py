"""Shared helpers of the GPU parity tests: run one batch through the HIP library and through the
CPU oracle on the same seeded inputs and compare tensor by tensor."""
from __future__ import annotations

import numpy as np

from paper_1911_05146_amd import workloads as W

TOL = {"bf16": 2e-2, "f32": 1e-4}     # max|gpu - ref| / max|ref| per tensor


def bf16_round(a: np.ndarray) -> np.ndarray:
    """float32 -> nearest-even bfloat16 -> float32 (what the device tensors will hold)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def device_inputs(spec, inp: W.StepInputs, mode: str):
    """Returns (StepInputs as seen by the device, in float32 for the oracle; torch device tensors)."""
    import torch
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if mode == "bf16" else torch.float32
    rnd = bf16_round if mode == "bf16" else (lambda a: a)
    act_host = [a if spec.has_stem else rnd(a) for a in inp.act_in]
    err_host = [rnd(e) for e in inp.err_in] if inp.err_in else None
    seen = W.StepInputs(inp.params, act_host, inp.labels, err_host)
    t = {
        "act_in": [torch.from_numpy(a).to(dev, torch.float32 if spec.has_stem else tdt) for a in act_host],
        "labels": [torch.from_numpy(l).to(dev) for l in inp.labels] if inp.labels else None,
        "err_in": [torch.from_numpy(e).to(dev, tdt) for e in err_host] if err_host else None,
    }
    return seen, t


def run_gpu_step(spec, inp: W.StepInputs, mode: str, multi_stream=False, sgd=None, part=None, keep=False):
    import torch
    from paper_1911_05146_amd import hpf
    seen, t = device_inputs(spec, inp, mode)
    own = part is None
    if own:
        part = hpf.Partition(spec, inp.params, hpf.HPF_BF16 if mode == "bf16" else hpf.HPF_F32)
    m = spec.num_microbatches
    streams = [torch.cuda.Stream() for _ in range(m)] if multi_stream else [None] * m
    torch.cuda.synchronize()
    part.loss.zero_()
    torch.cuda.synchronize()
    outs, errs = [], []
    for i in range(m):
        outs.append(part.forward_microbatch(i, t["act_in"][i], t["labels"][i] if t["labels"] else None,
                                            stream=streams[i]))
    for i in range(m):
        errs.append(part.backward_microbatch(i, t["err_in"][i] if t["err_in"] else None, stream=streams[i]))
    grad = part.grad_accum_read()
    torch.cuda.synchronize()
    res = {
        "act_out": [o.float().cpu().numpy() if o is not None else None for o in outs],
        "err_out": [e.float().cpu().numpy() if e is not None else None for e in errs],
        "loss": float(part.loss.item()),
        "grad": grad,
    }
    if sgd is not None:
        part.sgd_step(*sgd)
        res["params"] = part.params_read()
    if own and not keep:
        part.close()
    else:
        res["part"] = part
    return seen, res


def rel_err(got, ref):
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def compare(spec, res, ref, mode, what=("act_out", "err_out", "loss", "grad", "params"), tol=None):
    tol = TOL[mode] if tol is None else tol
    report = {}
    for k in what:
        if k not in ref or ref[k] is None or k not in res:
            continue
        if k in ("act_out", "err_out"):
            errs = [rel_err(g, r) for g, r in zip(res[k], ref[k]) if r is not None and g is not None]
            if errs:
                report[k] = max(errs)
        elif k == "loss":
            if spec.has_head:
                report[k] = abs(res[k] - ref[k]) / abs(ref[k])
        else:
            report[k] = rel_err(res[k], ref[k])
    bad = {k: v for k, v in report.items() if not (v <= tol)}
    assert not bad, f"{spec.name} [{mode}] over tolerance {tol}: {bad} (all: {report})"
    return report
