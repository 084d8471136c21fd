"""Teacher-forced parity, layer by layer.

End-to-end comparisons of a deep ReLU network say little once bf16 storage has let the two sides take
different ReLU decisions.  Here every layer is checked on its own instead: the tensors the device kept for
back-propagation (block inputs, convolution outputs, the partial errors of Eq. 5-7 of the paper at every
layer) are read back through hpf_stash_read, and each layer of the plain CPU oracle (float64, nothing
rounded) is fed the DEVICE's input of that layer.  Both sides then take every ReLU decision on the same
stored numbers, so every element of every tensor -- all blocks, all micro-batches, and every slice of the
accumulated gradient G -- must agree within the tolerance of one layer's rounding:
max|gpu - ref| / max|ref| <= 2e-2 (bf16 operands) or 1e-4 (fp32 check mode).

The only elements left out are explicit ReLU ties: pre-activations z whose magnitude is within the fp32
evaluation error of zero (the device evaluates z = x*scale + shift in fp32 from the same stored x, the
oracle in double); their number is reported and bounded.
"""
from __future__ import annotations

import numpy as np

from paper_1911_05146_amd import workloads as W

TOL = {"bf16": 2e-2, "f32": 1e-4}
STATS_TOL = {"bf16": 2e-4, "f32": 1e-9}
TIE_REL = {"bf16": 2e-5, "f32": 1e-12}    # |z| <= TIE_REL * (|gamma*xhat| + |beta|) + tiny: a tie


class Report:
    def __init__(self, mode):
        self.mode, self.tol = mode, TOL[mode]
        self.worst = {}          # tensor kind -> (err, where)
        self.bad = []
        self.n_elems = 0
        self.n_ties = 0
        self.n_tensors = 0

    def cmp(self, kind, where, got, ref, mask=None, tol=None):
        got = np.asarray(got, np.float64).ravel()
        ref = np.asarray(ref, np.float64).ravel()
        assert got.shape == ref.shape, (kind, where, got.shape, ref.shape)
        den = float(np.abs(ref).max()) or 1.0
        d = np.abs(got - ref)
        if mask is not None:
            d = d[~mask.ravel()]
        e = float(d.max() / den) if d.size else 0.0
        self.n_elems += d.size
        self.n_tensors += 1
        if e > self.worst.get(kind, (-1.0, ""))[0]:
            self.worst[kind] = (e, where)
        if not e <= (self.tol if tol is None else tol):
            self.bad.append((kind, where, e))
        return e

    def summary(self):
        parts = [f"{k} {v[0]:.2e}" for k, v in sorted(self.worst.items())]
        return (f"{self.n_tensors} tensors, {self.n_elems:.3e} elements, {self.n_ties} ReLU ties left out; worst "
                "max-norm error per tensor kind: " + ", ".join(parts))


def _f64(a):
    return np.ascontiguousarray(a, np.float64)


def _tie_mask(x, gamma, beta, mean, invstd, mode):
    xh = (x - mean) * invstd
    z = gamma * xh + beta
    return np.abs(z) <= TIE_REL[mode] * (np.abs(gamma * xh) + np.abs(beta)) + 1e-30


def layerwise_check(oracle, part, spec, seen, res, mode, eps=None, check_grad=True):
    """part: the hpf.Partition after a full batch (all forwards, all backwards, gradients not yet cleared).
    seen: StepInputs as the device saw them (float32 arrays of the rounded values); res: the outputs dict of
    parity.run_gpu_step.  Returns a Report; raises AssertionError on any element out of tolerance."""
    from paper_1911_05146_amd import hpf
    assert spec.first_from == 0 and spec.last_to == 0, "whole blocks only"
    assert spec.bn_mode == 0
    eps = spec.bn_eps if eps is None else eps
    rep = Report(mode)
    lay = {e.name: e for e in W.param_layout(spec)}
    params = _f64(seen.params)
    b, m, nb = spec.microbatch, spec.num_microbatches, len(spec.blocks)

    def P(name):
        e = lay[name]
        return params[e.offset:e.offset + e.size].reshape(e.shape)

    G = {name: np.zeros(e.shape, np.float64) for name, e in lay.items()}
    caller = lambda mb: {"act_in": seen.act_in[mb], "act_out": res["act_out"][mb],
                         "err_in": seen.err_in[mb] if seen.err_in else None, "err_out": res["err_out"][mb]}

    def rd(mb, unit, tensor, shape):
        t = part.stash_read(mb, unit, tensor)
        if isinstance(t, str):
            t = caller(mb)[t]
            assert t is not None, (unit, tensor)
        return _f64(t).reshape(shape)

    def bn(mb, unit, j, x, gname, bname, where):
        """Oracle BN+ReLU forward on the device's x; checks the device's statistics; returns a, mean, invstd."""
        g, bt = P(gname), P(bname)
        a, mean, invstd = oracle.bn_relu_fwd(x, g, bt, eps)
        st = part.stash_read(mb, unit, hpf.HPF_T_STATS0 + j)
        C = g.size
        # the mean in units of the channel's standard deviation
        rep.cmp("bn.mean", where, st[:C] * invstd, mean * invstd,
                tol=STATS_TOL[mode] * max(1.0, 1.0 / (float(np.abs(mean * invstd).max()) or 1.0)))
        rep.cmp("bn.invstd", where, st[C:], invstd, tol=STATS_TOL[mode])
        return a, mean, invstd, g, bt

    def bn_bwd(x, da, g, bt, mean, invstd, skip, gname, bname):
        dx, dg, db = oracle.bn_relu_bwd(x, da, g, bt, mean, invstd, skip=skip)
        G[gname] += dg
        G[bname] += db
        tie = _tie_mask(x, g, bt, mean, invstd, mode)
        rep.n_ties += int(tie.sum())
        return dx, tie

    loss = 0.0
    for mb in range(m):
        h, w = spec.in_h, spec.in_w
        if spec.has_stem:
            img = _f64(seen.act_in[mb])
            y = oracle.conv_fwd(img, P("stem.W"), 1)
            rep.cmp("stem.y", f"mb{mb}", rd(mb, -1, hpf.HPF_T_Y, y.shape), y)
            gy = rd(mb, -1, hpf.HPF_T_GY, y.shape)
            # the device's stem operand is the image as bfloat16 (im2col columns) in bf16 mode
            G["stem.W"] += oracle.conv_wgrad(img, gy, 3, 1)
        for i, blk in enumerate(spec.blocks):
            pre, tag = f"block{i}.", f"mb{mb} block{i}"
            ho, wo = h // blk.stride, w // blk.stride
            nconv = 2 if blk.kind == W.BASIC else 3
            R = (3, 3) if blk.kind == W.BASIC else (1, 3, 1)
            cin = (blk.c_in, blk.c_mid, blk.c_mid)
            x = rd(mb, i, hpf.HPF_T_X, (b, h, w, blk.c_in))
            ins = [x]
            for j in range(1, nconv):
                ins.append(rd(mb, i, hpf.HPF_T_C1 + j - 1, (b, ho, wo, cin[j])))
            y_dev = rd(mb, i, hpf.HPF_T_Y, (b, ho, wo, blk.c_out))
            a, st = [], []
            for j in range(nconv):
                aj, mean, invstd, g, bt = bn(mb, i, j, ins[j], pre + f"bn{j + 1}.gamma", pre + f"bn{j + 1}.beta", tag + f" bn{j + 1}")
                a.append(aj)
                st.append((mean, invstd, g, bt))
            shortcut = oracle.conv_fwd(a[0], P(pre + "Wproj"), blk.stride) if blk.has_proj else x
            for j in range(nconv):
                last = j == nconv - 1
                ref = oracle.conv_fwd(a[j], P(pre + f"W{j + 1}"), blk.stride if j == 0 else 1, add=shortcut if last else None)
                rep.cmp("fwd.y" if last else f"fwd.c{j + 1}", tag, y_dev if last else ins[j + 1], ref)
            # backward, every layer from the device's own incoming gradient
            gy = rd(mb, i, hpf.HPF_T_GY, y_dev.shape)
            d_out = [None] * nconv          # gradient w.r.t. the output of convolution j
            d_out[nconv - 1] = gy
            for j in range(nconv - 1):
                d_out[j] = rd(mb, i, hpf.HPF_T_DC1 + j, ins[j + 1].shape)
            gx_dev = rd(mb, i, hpf.HPF_T_GX, x.shape)
            for j in range(nconv - 1, -1, -1):
                Wj = P(pre + f"W{j + 1}")
                stride = blk.stride if j == 0 else 1
                G[pre + f"W{j + 1}"] += oracle.conv_wgrad(a[j], d_out[j], R[j], stride)
                da = oracle.conv_dgrad(d_out[j], Wj, ins[j].shape[1:3], stride)
                skip = None
                if j == 0:
                    if blk.has_proj:
                        G[pre + "Wproj"] += oracle.conv_wgrad(a[0], gy, 1, blk.stride)
                        da = da + oracle.conv_dgrad(gy, P(pre + "Wproj"), x.shape[1:3], blk.stride)
                    else:
                        skip = gy
                mean, invstd, g, bt = st[j]
                dx, tie = bn_bwd(ins[j], da, g, bt, mean, invstd, skip, pre + f"bn{j + 1}.gamma", pre + f"bn{j + 1}.beta")
                rep.cmp("bwd.gx" if j == 0 else f"bwd.dc{j}", tag, gx_dev if j == 0 else d_out[j - 1], dx, mask=tie)
            h, w = ho, wo
        if spec.has_head:
            c = spec.out_shape()[2]
            x = rd(mb, nb, hpf.HPF_T_X, (b, h, w, c))
            a, mean, invstd, g, bt = bn(mb, nb, 0, x, "head.bn.gamma", "head.bn.beta", f"mb{mb} head bn")
            l, gp, dl = oracle.head_fwd(a, P("head.Wfc"), P("head.bfc"), seen.labels[mb], spec.divisor)
            loss += l
            dwfc, dbfc, da = oracle.head_bwd(gp, dl, P("head.Wfc"), (h, w))
            G["head.Wfc"] += dwfc
            G["head.bfc"] += dbfc
            dx, tie = bn_bwd(x, da, g, bt, mean, invstd, None, "head.bn.gamma", "head.bn.beta")
            rep.cmp("bwd.head.gx", f"mb{mb}", rd(mb, nb, hpf.HPF_T_GX, x.shape), dx, mask=tie)
    if spec.has_head:
        rep.cmp("loss", "batch", [res["loss"]], [loss], tol=1e-3 if mode == "bf16" else 1e-5)
    if check_grad:
        gdev = np.asarray(res["grad"], np.float64)
        for name, e in lay.items():
            rep.cmp("G." + name.split(".", 1)[1] if name.startswith("block") else "G." + name, name,
                    gdev[e.offset:e.offset + e.size], G[name])
    total = max(rep.n_elems, 1)
    assert rep.n_ties <= 1e-4 * total + 10, f"{rep.n_ties} ReLU ties among {total} elements"
    assert not rep.bad, f"{spec.name} [{mode}] layer-wise parity failed ({len(rep.bad)} tensors), first: {rep.bad[:8]}; {rep.summary()}"
    return rep
