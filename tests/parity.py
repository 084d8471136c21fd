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


def run_gpu_step(spec, inp: W.StepInputs, mode: str, multi_stream=False, sgd=None, part=None, keep=False, grouped=False,
                 fusion=2):
    import torch
    from paper_1911_05146_amd import hpf
    seen, t = device_inputs(spec, inp, mode)
    own = part is None
    if own:
        part = hpf.Partition(spec, inp.params, hpf.HPF_BF16 if mode == "bf16" else hpf.HPF_F32)
        part.set_fusion(fusion)
    m = spec.num_microbatches
    streams = [torch.cuda.Stream() for _ in range(m)] if multi_stream else [None] * m
    torch.cuda.synchronize()
    part.loss.zero_()
    torch.cuda.synchronize()
    outs, errs = [], []
    if grouped:          # all micro-batches of the batch in one call per direction
        gs = torch.cuda.Stream()
        torch.cuda.synchronize()
        outs = part.forward_microbatches(0, t["act_in"], t["labels"], stream=gs) or [None] * m
        errs = part.backward_microbatches(0, m, t["err_in"], stream=gs) or [None] * m
    else:
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


def rel_l2(got, ref):
    ref = np.asarray(ref, np.float64).ravel()
    got = np.asarray(got, np.float64).ravel()
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / (den if den > 0 else 1.0))


def _tensors(res, spec):
    """The compared tensors of one batch: boundary tensors over all micro-batches, the loss, and the accumulated
    gradient / the parameters after the step split into the parameter tensors of the canonical layout."""
    out = {}
    for k in ("act_out", "err_out", "skip_out", "skip_err_out"):
        v = [t for t in res.get(k, []) if t is not None]
        if v:
            out[k] = np.concatenate([np.asarray(t, np.float64).ravel() for t in v])
    if spec.has_head:
        out["loss"] = np.array([res["loss"]], np.float64)
    for k in ("grad", "params"):
        if k in res:
            flat = np.asarray(res[k], np.float64)
            out[k] = flat
            for e in W.param_layout(spec):
                out[f"{k}:{e.name}"] = flat[e.offset:e.offset + e.size]
    return out


KAPPA = 1.1
FLOOR = {"bf16": 5e-3, "f32": 5e-3}
NOT_A_TEST = 0.5


def compare(spec, res, yard, mode, ref64=None, strict=False, tol=None, plain=None):
    """Parity of one batch, tensor by tensor (the gradient and the parameters also per parameter tensor).

    yard : the oracle run in the device's precision reading on the same inputs (float storage; in bf16 mode with
           the tensors the device keeps as bfloat16 rounded at the same points).
    plain: optionally the plain fp32 oracle (nothing rounded); the error against it is reported next to the other.
    Criterion A: max|gpu - yard| / max|yard| <= tol for the tensor (2e-2 bf16, 1e-4 fp32).  strict: A is required.
    Criterion B (sensitivity-limited), only for tensors that fail A and only if strict is False: a deep ReLU
           network's backward pass is discontinuous where a pre-activation is within rounding of 0, so two correct
           implementations of one precision reading scatter around the exact result by an amount the oracle
           itself can measure.  With ref64 the oracle in double and nothing rounded,
               relL2(gpu, ref64) <= (KAPPA + 3 / sqrt(2 n)) * relL2(yard, ref64) + FLOOR
           per tensor of n elements (KAPPA = 1.1: the two distances were measured equal to within 2 %; the second
           term is three standard deviations of a norm estimated from n samples, which matters for the
           per-channel tensors of 16 ... 128 elements).  A tensor for which the yardstick itself is at
           relL2 >= 0.5 of the exact result says nothing either way and fails the case as "not a test":
           such configurations are covered layer by layer instead (tests/teacher.py).
    A tensor the oracle returns and the device does not is a failure.  Returns {tensor: (criterion, error, ...)}.
    """
    tol = TOL[mode] if tol is None else tol
    g, y = _tensors(res, spec), _tensors(yard, spec)
    pl = _tensors(plain, spec) if plain is not None else None
    report, bad = {}, {}
    r64 = None
    for k in y:
        if k not in g:
            bad[k] = ("missing",)
            continue
        e = rel_err(g[k], y[k])
        if e <= tol:
            if ":" not in k:      # the per-parameter-tensor entries are only listed when they need criterion B
                report[k] = ("A", e) + ((rel_err(g[k], pl[k]),) if pl is not None else ())
            continue
        if k in ("grad", "params"):
            continue              # judged per parameter tensor below
        if strict or ref64 is None:
            bad[k] = ("A", e)
            continue
        if r64 is None:
            r64 = _tensors(ref64() if callable(ref64) else ref64, spec)
        eg, ey = rel_l2(g[k], r64[k]), rel_l2(y[k], r64[k])
        report[k] = ("B", e, eg, ey)
        if ey >= NOT_A_TEST:
            bad[k] = ("not a test: the yardstick is itself at relL2", ey)
        elif not eg <= (KAPPA + 3.0 / np.sqrt(2.0 * g[k].size)) * ey + FLOOR[mode]:
            bad[k] = ("B", e, eg, ey)
    assert not bad, f"{spec.name} [{mode}] parity failed: {bad} (passed: {report})"
    return report


def fmt(report):
    out, nb, worst = [], 0, None
    for k, v in report.items():
        if v[0] == "A":
            out.append(f"{k}: max-norm {v[1]:.2e}" + (f" (vs the plain fp32 oracle {v[2]:.2e})" if len(v) > 2 else ""))
        elif ":" in k:
            nb += 1
            if worst is None or v[2] / max(v[3], 1e-30) > worst[1][2] / max(worst[1][3], 1e-30):
                worst = (k, v)
        else:
            out.append(f"{k}: max-norm {v[1]:.2e} -> sensitivity-limited, relL2 gpu {v[2]:.2e} vs oracle-in-same-precision {v[3]:.2e}")
    if nb:
        k, v = worst
        out.append(f"{nb} parameter tensors sensitivity-limited, largest gpu/yardstick ratio at {k}: relL2 {v[2]:.2e} vs {v[3]:.2e}")
    return "; ".join(out)
