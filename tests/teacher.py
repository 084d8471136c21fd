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

import time

import numpy as np

from paper_1911_05146_amd import workloads as W

TOL = {"bf16": 2e-2, "f32": 1e-4}
STATS_TOL = {"bf16": 2e-4, "f32": 1e-9}
# A ReLU tie: |z| <= TIE_REL * (|gamma*xhat| + |beta|) + TIE_ABS * |gamma|.  The first term is the rounding of the
# device's fp32 evaluation of z, the second the difference between the device's statistics and the oracle's (the
# mean agrees to about 5e-7 standard deviations in bf16 mode, where the device reduces in fp32).
TIE_REL = {"bf16": 2e-5, "f32": 1e-12}
TIE_ABS = {"bf16": 2e-6, "f32": 1e-12}


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
    return np.abs(z) <= TIE_REL[mode] * (np.abs(gamma * xh) + np.abs(beta)) + TIE_ABS[mode] * np.abs(gamma)


def layerwise_check(oracle, part, spec, seen, res, mode, eps=None, check_grad=True):
    """part: the hpf.Partition after a full batch (all forwards, all backwards, gradients not yet cleared).
    seen: StepInputs as the device saw them (float32 arrays of the rounded values); res: the outputs dict of
    parity.run_gpu_step.  Returns a Report; raises AssertionError on any element out of tolerance."""
    from paper_1911_05146_amd import hpf
    assert spec.first_from == 0 and spec.last_to == 0, "whole blocks only"
    bn_mode = spec.bn_mode      # 1: frozen statistics (mean 0, variance 1)
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
        a, mean, invstd = oracle.bn_relu_fwd(x, g, bt, eps, mode=bn_mode)
        st = part.stash_read(mb, unit, hpf.HPF_T_STATS0 + j)
        C = g.size
        # the mean in units of the channel's standard deviation
        rep.cmp("bn.mean", where, st[:C] * invstd, mean * invstd,
                tol=STATS_TOL[mode] * max(1.0, 1.0 / (float(np.abs(mean * invstd).max()) or 1.0)))
        rep.cmp("bn.invstd", where, st[C:], invstd, tol=STATS_TOL[mode])
        return a, mean, invstd, g, bt

    Gabs = {}   # BatchNorm parameter gradients: sum of the absolute values of the terms (the scale of their rounding error)

    def bn_bwd(x, da, g, bt, mean, invstd, skip, gname, bname):
        dx, dg, db = oracle.bn_relu_bwd(x, da, g, bt, mean, invstd, mode=bn_mode, skip=skip)
        G[gname] += dg
        G[bname] += db
        tie = _tie_mask(x, g, bt, mean, invstd, mode)
        rep.n_ties += int(tie.sum())
        xh = (x - mean) * invstd
        dz = np.abs(da) * (g * xh + bt > 0)
        ax = tuple(range(x.ndim - 1))
        Gabs[bname] = Gabs.get(bname, 0.0) + dz.sum(axis=ax)
        Gabs[gname] = Gabs.get(gname, 0.0) + (dz * np.abs(xh)).sum(axis=ax)
        # a tie that falls the other way on the device moves these sums by up to its |da|
        Gabs[bname + ".tie"] = Gabs.get(bname + ".tie", 0.0) + (np.abs(da) * tie).sum(axis=ax)
        Gabs[gname + ".tie"] = Gabs.get(gname + ".tie", 0.0) + (np.abs(da * xh) * tie).sum(axis=ax)
        return dx, tie

    def stats_cmp(mb, unit, j, mean, invstd, where):
        st = part.stash_read(mb, unit, hpf.HPF_T_STATS0 + j)
        C = mean.size
        rep.cmp("bn.mean", where, st[:C] * invstd, mean * invstd,
                tol=STATS_TOL[mode] * max(1.0, 1.0 / (float(np.abs(mean * invstd).max()) or 1.0)))
        rep.cmp("bn.invstd", where, st[C:], invstd, tol=STATS_TOL[mode])

    def other_unit(mb, i, blk, h, w, pre, tag):
        """One unit of VGG-16 / ResNet-v1: every stored tensor of the forward pass from the device's stored input of
        its layer, and the gradient the unit hands on from the gradient it received (the gradients between its
        layers live in scratch memory on the device and are not kept; every ReLU decision inside the unit is taken
        on a stored tensor, the same on both sides).  Returns the unit's output height and width."""
        x = rd(mb, i, hpf.HPF_T_X, (b, h, w, blk.c_in))
        if blk.kind == W.DENSE:
            ho, wo = 1, 1
        else:
            ho, wo = h // blk.stride, w // blk.stride
        y_dev = rd(mb, i, hpf.HPF_T_Y, (b, ho, wo, blk.c_out))
        gy = rd(mb, i, hpf.HPF_T_GY, y_dev.shape)
        gx_dev = rd(mb, i, hpf.HPF_T_GX, x.shape)
        taint = None
        if blk.kind == W.POSTACT:
            c1 = rd(mb, i, hpf.HPF_T_C1, (b, ho, wo, blk.c_mid))
            try:
                a1 = rd(mb, i, hpf.HPF_T_A0, c1.shape)
            except hpf.HpfError:
                a1 = None       # inside an image-resident run relu(bn1(c1)) never reaches memory
            c2 = rd(mb, i, hpf.HPF_T_C2, y_dev.shape)
            W1, W2 = P(pre + "W1"), P(pre + "W2")
            g1, b1, g2, b2 = (P(pre + n) for n in ("bn1.gamma", "bn1.beta", "bn2.gamma", "bn2.beta"))
            rep.cmp("fwd.c1", tag, c1, oracle.conv_fwd(x, W1, blk.stride))
            a1_ref, mean1, inv1 = oracle.bn_relu_fwd(c1, g1, b1, eps, mode=bn_mode)
            stats_cmp(mb, i, 0, mean1, inv1, tag + " bn1")
            if a1 is None:
                a1 = a1_ref     # the device applied the same map to the same stored c1 while staging
            else:
                rep.cmp("fwd.a1", tag, a1, a1_ref)
            rep.cmp("fwd.c2", tag, c2, oracle.conv_fwd(a1, W2, 1))
            if blk.has_proj:
                sc = rd(mb, i, hpf.HPF_T_SC, y_dev.shape)
                rep.cmp("fwd.shortcut", tag, sc, oracle.conv_fwd(x, P(pre + "Wproj"), blk.stride))
            else:
                sc = x
            y_ref, mean2, inv2 = oracle.bn_add_relu_fwd(c2, g2, b2, sc, eps, mode=bn_mode)
            stats_cmp(mb, i, 1, mean2, inv2, tag + " bn2")
            rep.cmp("fwd.y", tag, y_dev, y_ref)
            dc2, dz, dg2, db2 = oracle.bn_add_relu_bwd(c2, y_dev, gy, g2, mean2, inv2, mode=bn_mode)
            G[pre + "bn2.gamma"] += dg2
            G[pre + "bn2.beta"] += db2
            G[pre + "W2"] += oracle.conv_wgrad(a1, dc2, 3, 1)
            da1 = oracle.conv_dgrad(dc2, W2, (ho, wo), 1)
            dc1, tie = bn_bwd(c1, da1, g1, b1, mean1, inv1, None, pre + "bn1.gamma", pre + "bn1.beta")
            G[pre + "W1"] += oracle.conv_wgrad(x, dc1, 3, blk.stride)
            gx = oracle.conv_dgrad(dc1, W1, (h, w), blk.stride)
            if blk.has_proj:
                G[pre + "Wproj"] += oracle.conv_wgrad(x, dz, 1, blk.stride)
                gx = gx + oracle.conv_dgrad(dz, P(pre + "Wproj"), (h, w), blk.stride)
            else:
                gx = gx + dz
            taint = np.broadcast_to(_spread(oracle, tie.any(axis=-1), 3, blk.stride, (h, w))[..., None], gx.shape)
        elif blk.kind == W.CONV_RELU:
            Wc, bias = P(pre + "W"), P(pre + "bias")
            y0 = rd(mb, i, hpf.HPF_T_Y0, (b, h, w, blk.c_out)) if blk.stride == 2 else y_dev
            rep.cmp("fwd.conv_relu", tag, y0, oracle.bias_act_fwd(oracle.conv_fwd(x, Wc, 1), bias, True))
            d0 = gy
            if blk.stride == 2:
                rep.cmp("fwd.pool", tag, y_dev, oracle.maxpool2_fwd(y0), tol=0.0)       # a selection: exact
                d0 = oracle.maxpool2_bwd(y0, gy)
            dz, db = oracle.bias_act_bwd(y0, d0, True)
            G[pre + "bias"] += db
            G[pre + "W"] += oracle.conv_wgrad(x, dz, 3, 1)
            gx = oracle.conv_dgrad(dz, Wc, (h, w), 1)
        elif blk.kind == W.DENSE:
            K = h * w * blk.c_in
            W4, bias = P(pre + "W").reshape(1, 1, K, blk.c_out), P(pre + "bias")
            xr = x.reshape(b, 1, 1, K)
            rep.cmp("fwd.dense", tag, y_dev, oracle.bias_act_fwd(oracle.conv_fwd(xr, W4, 1), bias, blk.c_mid != 0))
            dz, db = oracle.bias_act_bwd(y_dev, gy, blk.c_mid != 0)
            G[pre + "bias"] += db
            G[pre + "W"] += oracle.conv_wgrad(xr, dz, 1, 1).reshape(K, blk.c_out)
            gx = oracle.conv_dgrad(dz, W4, (1, 1), 1).reshape(x.shape)
        elif blk.kind == W.BN_RELU:
            g, bt = P(pre + "bn.gamma"), P(pre + "bn.beta")
            a_ref, mean, invstd = oracle.bn_relu_fwd(x, g, bt, eps, mode=bn_mode)
            stats_cmp(mb, i, 0, mean, invstd, tag + " bn")
            rep.cmp("fwd.bn_relu", tag, y_dev, a_ref)
            gx, taint = bn_bwd(x, gy, g, bt, mean, invstd, None, pre + "bn.gamma", pre + "bn.beta")
        else:
            bias = P(pre + "bias")
            rep.cmp("fwd.bias_relu", tag, y_dev, oracle.bias_act_fwd(x, bias, True))
            gx, db = oracle.bias_act_bwd(y_dev, gy, True)
            G[pre + "bias"] += db
        rep.cmp("bwd.gx", tag, gx_dev, gx, mask=taint)
        return ho, wo

    loss = 0.0
    t_last = time.time()
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
            if time.time() - t_last > 30:      # a long run says where it is
                print(f"  ... layer-wise {spec.name}: micro-batch {mb}, block {i}", flush=True)
                t_last = time.time()
            pre, tag = f"block{i}.", f"mb{mb} block{i}"
            if not blk.residual:
                h, w = other_unit(mb, i, blk, h, w, pre, tag)
                continue
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
            head_bn = getattr(spec, "head_bn", True)
            if head_bn:
                a, mean, invstd, g, bt = bn(mb, nb, 0, x, "head.bn.gamma", "head.bn.beta", f"mb{mb} head bn")
            else:
                a = x
            l, gp, dl = oracle.head_fwd(a, P("head.Wfc"), P("head.bfc"), seen.labels[mb], spec.divisor)
            loss += l
            dwfc, dbfc, da = oracle.head_bwd(gp, dl, P("head.Wfc"), (h, w))
            G["head.Wfc"] += dwfc
            G["head.bfc"] += dbfc
            dx, tie = bn_bwd(x, da, g, bt, mean, invstd, None, "head.bn.gamma", "head.bn.beta") if head_bn else (da, None)
            rep.cmp("bwd.head.gx", f"mb{mb}", rd(mb, nb, hpf.HPF_T_GX, x.shape), dx, mask=tie)
    if spec.has_head:
        rep.cmp("loss", "batch", [res["loss"]], [loss], tol=1e-3 if mode == "bf16" else 1e-5)
    if check_grad:
        gdev = np.asarray(res["grad"], np.float64)
        for name, e in lay.items():
            kind = "G." + name.split(".", 1)[1] if name.startswith("block") else "G." + name
            got, ref = gdev[e.offset:e.offset + e.size], G[name].ravel()
            if name in Gabs and not np.abs(got - ref).max() <= rep.tol * (np.abs(ref).max() or 1.0):
                # A sum over M terms of both signs can come out far smaller than its terms; what rounding can do
                # to it scales with the sum of the terms' magnitudes, not with the result.  Such a slice passes if
                # every element is within that bound: one bf16 rounding per term (2^-8), plus the ties.
                bound = 2.0 ** -8 * Gabs[name] + Gabs[name + ".tie"]
                ok = bool((np.abs(got - ref) <= bound).all())
                print(f"[note] {spec.name} {name}: max-norm {np.abs(got - ref).max() / (np.abs(ref).max() or 1.0):.3e} over {ref.size} "
                      f"channels; |err| / (2^-8 sum|terms| + ties) <= {float((np.abs(got - ref) / bound).max()):.3f}; "
                      f"max|ref| {np.abs(ref).max():.3e}, sum|terms| {Gabs[name].max():.3e}, ties {Gabs[name + '.tie'].max():.3e}", flush=True)
                rep.cmp(kind + ".cancelling", name, got, ref, tol=np.inf if ok else 0.0)
                continue
            rep.cmp(kind, name, got, ref)
    total = max(rep.n_elems, 1)
    assert rep.n_ties <= 1e-4 * total + 10, f"{rep.n_ties} ReLU ties among {total} elements"
    if rep.bad:
        print(f"[layer-wise FAILED] {spec.name} [{mode}]: {rep.bad[:12]} ({len(rep.bad)})", flush=True)
    assert not rep.bad, f"{spec.name} [{mode}] layer-wise parity failed ({len(rep.bad)} tensors), first: {rep.bad[:8]}; {rep.summary()}"
    return rep


# ---------------------------------------------------------------------------------------------------------
# Block by block: one block of cascade, with an explicit mask of the ReLU decisions that differ
# ---------------------------------------------------------------------------------------------------------
def _spread(oracle, pix, R, stride, in_hw):
    """Pixels of a convolution's input that receive gradient from the marked output pixels (the oracle's own
    data-gradient geometry applied to an indicator)."""
    if not pix.any():
        return np.zeros((pix.shape[0],) + tuple(in_hw), bool)
    ind = np.ascontiguousarray(pix[..., None], np.float64)
    return oracle.conv_dgrad(ind, np.ones((R, R, 1, 1)), in_hw, stride)[..., 0] > 0


def blockwise_check(oracle, part, spec, seen, res, mode, frac_ok=0.9, l2_ok=0.15):
    """Every block from the device's block input x_k and incoming gradient gy_k alone: the plain oracle (float64,
    nothing rounded) runs the whole block -- its own c1, c2, its own ReLU decisions -- and every tensor of the
    block is compared element by element.  Inside one block the device's c1 / c2 differ from the oracle's by
    bf16 rounding, so a few ReLU decisions of BatchNorm 2 / 3 fall the other way; these are found explicitly
    (decision from the device's stored tensor vs decision of the oracle, both evaluated in double; the forward
    comparison bounds how far from zero such a pre-activation can be), and only the gradient elements that such a decision can
    reach through the block's own layers are left out.  Every other element must be within tolerance.
    Over ALL elements of a gradient tensor the agreement is statistical by nature -- a fraction f of differing
    decisions alone gives a relative L2 distance of about sqrt(2 f), 0.05 for the measured f = 0.14 % -- so there
    only sanity bounds apply (at least frac_ok of the elements within tolerance, relative L2 distance below
    l2_ok); the measured figures are reported, and so is the largest share of a tensor that had to be left out:
    every element of a gradient behind a 3x3 convolution of 256 channels is within reach of some differing
    decision, so for wide blocks the strict statement is the layer-wise one."""
    from paper_1911_05146_amd import hpf
    assert spec.first_from == 0 and spec.last_to == 0 and spec.bn_mode == 0
    assert all(blk.residual for blk in spec.blocks), "block-wise: pre-activation residual blocks only"
    rep = Report(mode)
    tol = rep.tol
    lay = {e.name: e for e in W.param_layout(spec)}
    params = _f64(seen.params)
    b, m = spec.microbatch, spec.num_microbatches
    P = lambda name: params[lay[name].offset:lay[name].offset + lay[name].size].reshape(lay[name].shape)
    G = {name: np.zeros(e.shape, np.float64) for name, e in lay.items() if name.startswith("block")}
    caller = lambda mb: {"act_in": seen.act_in[mb], "act_out": res["act_out"][mb],
                         "err_in": seen.err_in[mb] if seen.err_in else None, "err_out": res["err_out"][mb]}

    def rd(mb, unit, tensor, shape):
        t = part.stash_read(mb, unit, tensor)
        if isinstance(t, str):
            t = caller(mb)[t]
        return _f64(t).reshape(shape)

    n_flips = n_masked = 0
    worst_frac, worst_l2, worst_taint = 1.0, 0.0, 0.0

    def cmp_masked(kind, where, got, ref, taint):
        nonlocal n_masked, worst_frac, worst_l2, worst_taint
        rep.cmp(kind, where, got, ref, mask=taint)                 # every element no differing decision can reach
        den = float(np.abs(ref).max()) or 1.0
        frac = float((np.abs(got - ref) <= tol * den).mean())      # ... and nearly all elements altogether
        l2 = float(np.linalg.norm((got - ref).ravel()) / (np.linalg.norm(ref.ravel()) or 1.0))
        worst_frac, worst_l2 = min(worst_frac, frac), max(worst_l2, l2)
        n_masked += int(taint.sum()) if taint is not None else 0
        worst_taint = max(worst_taint, float(taint.mean()) if taint is not None else 0.0)
        if frac < frac_ok or l2 > l2_ok:
            rep.bad.append((kind + ".all", where, (frac, l2)))

    t_last = time.time()
    for mb in range(m):
        h, w = spec.in_h, spec.in_w
        for i, blk in enumerate(spec.blocks):
            if time.time() - t_last > 30:
                print(f"  ... block-wise {spec.name}: micro-batch {mb}, block {i}", flush=True)
                t_last = time.time()
            pre, tag = f"block{i}.", f"mb{mb} block{i}"
            ho, wo = h // blk.stride, w // blk.stride
            nconv = 2 if blk.kind == W.BASIC else 3
            R = (3, 3) if blk.kind == W.BASIC else (1, 3, 1)
            x = rd(mb, i, hpf.HPF_T_X, (b, h, w, blk.c_in))
            gy = rd(mb, i, hpf.HPF_T_GY, (b, ho, wo, blk.c_out))
            ins, a, st, flips = [x], [], [], []
            for j in range(nconv):
                g, bt = P(pre + f"bn{j + 1}.gamma"), P(pre + f"bn{j + 1}.beta")
                aj, mean, invstd = oracle.bn_relu_fwd(ins[j], g, bt, spec.bn_eps)
                a.append(aj)
                st.append((mean, invstd, g, bt))
                if j == 0:
                    flips.append(np.zeros(x.shape, bool))      # same x on both sides
                else:                                          # the device decides on its own stored c_j and statistics
                    cdev = rd(mb, i, hpf.HPF_T_C1 + j - 1, ins[j].shape)
                    sd = part.stash_read(mb, i, hpf.HPF_T_STATS0 + j)
                    C = g.size
                    z_ref = g * ((ins[j] - mean) * invstd) + bt
                    z_dev = g * ((cdev - sd[:C]) * sd[C:]) + bt
                    f = (z_ref > 0) != (z_dev > 0)
                    # (a decision can only differ where |z_ref| <= |z_ref - z_dev|, and the forward comparison just
                    # below bounds that difference: every differing decision is a near-tie by construction)
                    flips.append(f)
                    n_flips += int(f.sum())
                    rep.cmp(f"fwd.c{j}", tag, cdev, ins[j])
                if j + 1 < nconv:
                    ins.append(oracle.conv_fwd(aj, P(pre + f"W{j + 1}"), blk.stride if j == 0 else 1))
            shortcut = oracle.conv_fwd(a[0], P(pre + "Wproj"), blk.stride) if blk.has_proj else x
            y = oracle.conv_fwd(a[-1], P(pre + f"W{nconv}"), blk.stride if nconv == 1 else 1, add=shortcut)
            rep.cmp("fwd.y", tag, rd(mb, i, hpf.HPF_T_Y, y.shape), y)
            # backward from gy with the oracle's own intermediates
            d = gy
            taint_pix = np.zeros((b, ho, wo), bool)            # pixels of the current gradient tensor a flip can reach
            for j in range(nconv - 1, -1, -1):
                stride = blk.stride if j == 0 else 1
                G[pre + f"W{j + 1}"] += oracle.conv_wgrad(a[j], d, R[j], stride)
                da = oracle.conv_dgrad(d, P(pre + f"W{j + 1}"), ins[j].shape[1:3], stride)
                taint_pix = _spread(oracle, taint_pix, R[j], stride, ins[j].shape[1:3])
                skip = None
                if j == 0:
                    if blk.has_proj:
                        G[pre + "Wproj"] += oracle.conv_wgrad(a[0], gy, 1, blk.stride)
                        da = da + oracle.conv_dgrad(gy, P(pre + "Wproj"), x.shape[1:3], blk.stride)
                    else:
                        skip = gy
                mean, invstd, g, bt = st[j]
                dx, dg, db = oracle.bn_relu_bwd(ins[j], da, g, bt, mean, invstd, skip=skip)
                G[pre + f"bn{j + 1}.gamma"] += dg
                G[pre + f"bn{j + 1}.beta"] += db
                taint = taint_pix[..., None] | flips[j] | _tie_mask(ins[j], g, bt, mean, invstd, mode)
                dev = rd(mb, i, hpf.HPF_T_GX if j == 0 else hpf.HPF_T_DC1 + j - 1, dx.shape)
                cmp_masked("bwd.gx" if j == 0 else f"bwd.dc{j}", tag, dev, dx, taint)
                taint_pix = taint.any(axis=-1)
                d = dx
            h, w = ho, wo
    gdev = np.asarray(res["grad"], np.float64)
    for name in G:
        e = lay[name]
        got, ref = gdev[e.offset:e.offset + e.size], G[name].ravel()
        l2 = float(np.linalg.norm(got - ref) / (np.linalg.norm(ref) or 1.0))
        worst_l2 = max(worst_l2, l2)
        rep.worst["G.relL2"] = max(rep.worst.get("G.relL2", (0.0, "")), (l2, name))
        if l2 > l2_ok:
            rep.bad.append(("G.relL2", name, l2))
    rep.n_ties = n_flips
    rep.extra = (f"{n_flips} differing ReLU decisions (all near-ties), {n_masked} gradient elements within their reach left out (at most {worst_taint:.0%} of a tensor); "
                 f"over ALL elements: >= {worst_frac:.5f} of every tensor within tolerance, worst relative L2 {worst_l2:.2e}")
    if rep.bad:
        print(f"[block-wise FAILED] {spec.name} [{mode}]: {rep.bad[:12]} ({len(rep.bad)}); {rep.extra}", flush=True)
    assert not rep.bad, f"{spec.name} [{mode}] block-wise parity failed ({len(rep.bad)}), first: {rep.bad[:8]}; {rep.summary()}; {rep.extra}"
    return rep


def run_and_check(oracle, spec, mode, grouped=False, fusion=2, multi_stream=False, randomize_affine=True, blockwise=True,
                  beta_shift=0.0):
    """One batch on the device, then the layer-wise and (optionally) the block-wise check.  For a partition of a
    single block the block-wise check IS the end-to-end comparison of err_out and G against the plain oracle, with
    the differing ReLU decisions found explicitly instead of re-drawing the inputs until none occurs."""
    from parity import run_gpu_step
    inp = W.make_inputs(spec, randomize_affine=randomize_affine)
    if beta_shift:
        for e in W.param_layout(spec):
            if e.kind == "beta":
                inp.params[e.offset:e.offset + e.size] += beta_shift
    seen, res = run_gpu_step(spec, inp, mode, grouped=grouped, fusion=fusion, multi_stream=multi_stream, keep=True)
    part = res.pop("part")
    try:
        rep = layerwise_check(oracle, part, spec, seen, res, mode)
        print(f"[layer-wise] {spec.name} {mode}: {rep.summary()}", flush=True)
        if blockwise:
            rb = blockwise_check(oracle, part, spec, seen, res, mode)
            print(f"[block-wise] {spec.name} {mode}: {rb.summary()}; {rb.extra}", flush=True)
    finally:
        part.close()
    return rep
