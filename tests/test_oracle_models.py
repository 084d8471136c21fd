"""Pins for the oracle's units of the paper's two other models (no GPU): the post-activation basic block of
ResNet-110-v1 and the layers of VGG-16 (paper Section "Model-Parallelism on a Single Node"; layer types:
Section "Background").

Every gradient against central finite differences in double (every single parameter, sampled inputs); the
forward wiring against an independent numpy / scipy composition; max-pool and bias + ReLU against closed
forms; partition equivalence (the paper's premise) for both models; parameter counts of the published
architectures (ResNet-110: 1.7 M; VGG-16's 13 convolutions: 14.7 M).
"""
import numpy as np
import pytest

from paper_1911_05146_amd import workloads as W
from test_oracle_partition import np_conv, replace_params, scalar_objective, tiny

FD_CASES = {
    "postact_identity": dict(blocks=[W.Block(W.POSTACT, 3, 3, 3, 1)]),
    "postact_stride2_proj": dict(blocks=[W.Block(W.POSTACT, 2, 4, 4, 2), W.Block(W.POSTACT, 4, 4, 4, 1)]),
    "conv_relu_pool": dict(blocks=[W.Block(W.CONV_RELU, 2, 3, 3, 1), W.Block(W.CONV_RELU, 3, 4, 4, 2)]),
    "dense_relu_dense": dict(blocks=[W.Block(W.DENSE, 2, 1, 5, 1), W.Block(W.DENSE, 5, 0, 3, 1)], in_hw=2),
    "bn_relu_and_bias_relu_units": dict(blocks=[W.Block(W.BN_RELU, 3, 3, 3, 1), W.Block(W.BIAS_RELU, 3, 3, 3, 1)]),
    "resnet_v1_tiny": dict(blocks=[W.Block(W.BN_RELU, 3, 3, 3, 1), W.Block(W.POSTACT, 3, 3, 3, 1), W.Block(W.POSTACT, 3, 4, 4, 2)],
                           stem=True, head=True, head_bn=False),
    "vgg_tiny": dict(blocks=[W.Block(W.BIAS_RELU, 3, 3, 3, 1), W.Block(W.CONV_RELU, 3, 3, 3, 2), W.Block(W.CONV_RELU, 3, 4, 4, 2),
                             W.Block(W.DENSE, 4, 1, 6, 1)], stem=True, head=True, head_bn=False),
}


@pytest.mark.parametrize("case", sorted(FD_CASES))
def test_gradients_match_finite_differences(oracle, case):
    spec = tiny(**FD_CASES[case])
    inp = W.make_inputs(spec, randomize_affine=True)
    params = inp.params.astype(np.float64)
    inp.act_in = [a.astype(np.float64) for a in inp.act_in]
    res = oracle.run_step(spec, replace_params(inp, params), np.float64)
    G = res["grad"]
    h = 1e-6
    f = lambda p, a=None: scalar_objective(oracle, spec, inp, p, a)
    scale = max(np.abs(G).max(), 1.0)
    bad = [i for i in range(params.size)
           if abs((f(params + h * np.eye(1, params.size, i)[0]) - f(params - h * np.eye(1, params.size, i)[0])) / (2 * h) - G[i]) > 1e-6 * scale]
    assert not bad, f"{len(bad)} of {params.size} parameter gradients off: {bad[:10]}"
    if not spec.has_stem:                                # err_out = d objective / d act_in
        scale = max(max(np.abs(e).max() for e in res["err_out"]), 1.0)
        rs = np.random.default_rng(3)
        for _ in range(40):
            mb = int(rs.integers(spec.num_microbatches))
            idx = tuple(int(rs.integers(s)) for s in inp.act_in[0].shape)
            ap, am = [a.copy() for a in inp.act_in], [a.copy() for a in inp.act_in]
            ap[mb][idx] += h
            am[mb][idx] -= h
            fd = (f(params, ap) - f(params, am)) / (2 * h)
            assert abs(fd - res["err_out"][mb][idx]) <= 1e-6 * scale


def np_bn(x, g, b, eps):
    m, v = x.mean((0, 1, 2)), x.var((0, 1, 2))
    return g * (x - m) / np.sqrt(v + eps) + b


def np_forward(spec, params, x, labels):
    """The same models composed from numpy / scipy pieces (correlate2d, mean / var, reshape-max, matmul)."""
    P = {e.name: params[e.offset:e.offset + e.size].reshape(e.shape) for e in W.param_layout(spec)}
    if spec.has_stem:
        x = np_conv(x, P["stem.W"], 1)
    for i, b in enumerate(spec.blocks):
        p = f"block{i}."
        if b.kind == W.POSTACT:
            a1 = np.maximum(np_bn(np_conv(x, P[p + "W1"], b.stride), P[p + "bn1.gamma"], P[p + "bn1.beta"], spec.bn_eps), 0)
            z2 = np_bn(np_conv(a1, P[p + "W2"], 1), P[p + "bn2.gamma"], P[p + "bn2.beta"], spec.bn_eps)
            x = np.maximum(z2 + (np_conv(x, P[p + "Wproj"], b.stride) if b.has_proj else x), 0)
        elif b.kind == W.CONV_RELU:
            x = np.maximum(np_conv(x, P[p + "W"], 1) + P[p + "bias"], 0)
            if b.stride == 2:
                n, h, w, c = x.shape
                x = x.reshape(n, h // 2, 2, w // 2, 2, c).max(axis=(2, 4))
        elif b.kind == W.DENSE:
            x = x.reshape(x.shape[0], -1) @ P[p + "W"] + P[p + "bias"]
            x = (np.maximum(x, 0) if b.c_mid else x)[:, None, None, :]
        elif b.kind == W.BN_RELU:
            x = np.maximum(np_bn(x, P[p + "bn.gamma"], P[p + "bn.beta"], spec.bn_eps), 0)
        else:
            x = np.maximum(x + P[p + "bias"], 0)
    if not spec.has_head:
        return x
    logits = x.mean((1, 2)) @ P["head.Wfc"] + P["head.bfc"]
    from scipy.special import logsumexp
    return np.sum(logsumexp(logits, axis=1) - logits[np.arange(len(labels)), labels]) / spec.divisor


@pytest.mark.parametrize("case", ["postact_stride2_proj", "conv_relu_pool", "dense_relu_dense", "resnet_v1_tiny", "vgg_tiny"])
def test_forward_matches_numpy_composition(oracle, case):
    spec = tiny(**dict({"in_hw": 8}, **FD_CASES[case]))
    inp = W.make_inputs(spec, randomize_affine=True)
    params = inp.params.astype(np.float64)
    part = oracle.OraclePartition(spec, params, np.float64)
    tot = 0.0
    for i in range(spec.num_microbatches):
        x = inp.act_in[i].astype(np.float64)
        out = part.forward(i, x, inp.labels[i] if inp.labels else None)
        ref = np_forward(spec, params, x, inp.labels[i] if inp.labels else None)
        if spec.has_head:
            tot += ref
        else:
            assert np.abs(out - ref).max() < 1e-11
    if spec.has_head:
        assert abs(part.loss[0] - tot) < 1e-12


def test_maxpool_closed_forms(oracle):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 6, 8, 5))
    y = oracle.maxpool2_fwd(x)
    assert np.array_equal(y, x.reshape(3, 3, 2, 4, 2, 5).max(axis=(2, 4)))
    dy = rng.standard_normal(y.shape)
    dx = oracle.maxpool2_bwd(x, dy)
    win = dx.reshape(3, 3, 2, 4, 2, 5)
    assert np.array_equal(win.sum(axis=(2, 4)), dy)                       # all of a window's gradient arrives ...
    assert np.array_equal((win != 0).sum(axis=(2, 4)), (dy != 0) * 1)     # ... at one position ...
    assert np.all((dx == 0) | (np.repeat(np.repeat(y, 2, 1), 2, 2) == x))  # ... which holds the maximum
    # equal maxima: the first in row-major order takes it
    t = np.zeros((1, 2, 2, 1))
    assert np.array_equal(oracle.maxpool2_bwd(t, np.ones((1, 1, 1, 1))).ravel(), [1, 0, 0, 0])
    t[0, 0, 1, 0] = t[0, 1, 0, 0] = 2.0
    assert np.array_equal(oracle.maxpool2_bwd(t, np.ones((1, 1, 1, 1))).ravel(), [0, 1, 0, 0])


def test_bias_relu_and_join_closed_forms(oracle):
    rng = np.random.default_rng(6)
    x, bias = rng.standard_normal((2, 3, 3, 4)), rng.standard_normal(4)
    y = oracle.bias_act_fwd(x, bias, relu=True)
    assert np.allclose(y, np.maximum(x + bias, 0), atol=0, rtol=1e-15)
    assert np.allclose(oracle.bias_act_fwd(x, bias, relu=False), x + bias, atol=0, rtol=1e-15)
    dy = rng.standard_normal(x.shape)
    dx, db = oracle.bias_act_bwd(y, dy, relu=True)
    assert np.array_equal(dx, dy * (y > 0)) and np.allclose(db, (dy * (y > 0)).sum((0, 1, 2)))
    dx, db = oracle.bias_act_bwd(y, dy, relu=False)
    assert np.array_equal(dx, dy) and np.allclose(db, dy.sum((0, 1, 2)))
    # the residual join of the post-activation block: statistics of x only, the shortcut enters after the normalisation
    g, b, add = rng.uniform(0.5, 1.5, 4), rng.standard_normal(4), rng.standard_normal(x.shape)
    yj, mean, invstd = oracle.bn_add_relu_fwd(x, g, b, add)
    assert np.allclose(mean, x.mean((0, 1, 2))) and np.allclose(invstd, 1 / np.sqrt(x.var((0, 1, 2)) + 1e-5))
    assert np.allclose(yj, np.maximum(np_bn(x, g, b, 1e-5) + add, 0), atol=1e-14)
    dxj, dadd, dg, dbt = oracle.bn_add_relu_bwd(x, yj, dy, g, mean, invstd)
    dz = dy * (yj > 0)
    assert np.array_equal(dadd, dz) and np.allclose(dbt, dz.sum((0, 1, 2))) and np.allclose(dg, (dz * (x - mean) * invstd).sum((0, 1, 2)))
    xh = (x - mean) * invstd
    assert np.abs(dxj.sum((0, 1, 2))).max() < 1e-12                       # the BatchNorm backward removes the mean ...
    assert np.allclose((dxj * xh).sum((0, 1, 2)), g * invstd * dg * 1e-5 * invstd ** 2, rtol=1e-9, atol=1e-14)   # ... and, up to eps, the xhat component


@pytest.mark.parametrize("model", ["resnet_v1", "vgg16"])
def test_partition_chain_equals_unsplit_model(oracle, model):
    """The paper's premise for its two other models: cut into partitions and run micro-batch by micro-batch, the
    model computes what the unsplit model computes (bitwise in the oracle: same operations in the same order)."""
    b, m = 2, 2
    if model == "resnet_v1":
        mk = lambda n, p: W.resnet110_v1(n, p, microbatch=b, num_microbatches=m, n_per_stage=2)
    else:
        mk = lambda n, p: W.vgg16(n, p, microbatch=b, num_microbatches=m, widths=(4, 8, 8, 8, 8), dense=(16, 16))
    whole = mk(1, 0)
    inp = W.make_inputs(whole, randomize_affine=True)
    ref = oracle.run_step(whole, inp, np.float64)
    for n_parts in (2, 4):
        specs = [mk(n_parts, p) for p in range(n_parts)]
        assert sum(W.n_params(s) for s in specs) == W.n_params(whole)
        parts, off = [], 0
        for s in specs:
            parts.append(oracle.OraclePartition(s, inp.params[off:off + W.n_params(s)], np.float64))
            off += W.n_params(s)
        for i in range(m):
            x = inp.act_in[i].astype(np.float64)
            for s, part in zip(specs, parts):
                x = part.forward(i, x, inp.labels[i] if s.has_head else None)
        for i in range(m):
            e = None
            for s, part in zip(reversed(specs), reversed(parts)):
                e = part.backward(i, e, want_err_out=not s.has_stem)
        assert float(parts[-1].loss[0]) == ref["loss"]
        assert np.array_equal(np.concatenate([p.grad() for p in parts]), ref["grad"])


def test_parameter_counts_of_the_published_architectures():
    assert W.n_params(W.resnet110_v1()) == 1730522            # "1.7 M" for ResNet-110 on 32x32 images
    v = W.vgg16()
    convs = sum(e.size for e in W.param_layout(v) if e.kind == "conv" or (e.kind == "bias" and ".bias" in e.name and len(e.shape) == 1
                                                                         and e.name.split(".")[0] in [f"block{i}" for i in range(13)]))
    assert convs == 14714688                                  # the 13 convolutions with their biases: 14.7 M
    assert len([b for b in v.blocks if b.kind in (W.CONV_RELU,)]) + 1 == 13 and len([b for b in v.blocks if b.kind == W.DENSE]) == 2
