"""Pins for the CPU oracle's single operations (no GPU).

Every check compares the oracle with something that is not the oracle: a library
routine (numpy matmul, scipy correlate2d, numpy mean/var), a closed form, an
algebraic identity, or a hand-worked fixture.  Citations: convolution layers,
back-propagation with partial errors -- paper Section "Implementing Distributed
Back-Propagation", Eq. 1-7.
"""
import os

import numpy as np
import pytest
from scipy.signal import correlate2d

rng = np.random.default_rng(7)


def rnd(*shape):
    return rng.standard_normal(shape)


# ------------------------------------------------------------------ conv forward
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_conv1x1_is_matmul(oracle, dtype):
    x = rnd(3, 5, 4, 6).astype(dtype)
    w = rnd(1, 1, 6, 7).astype(dtype)
    y = oracle.conv_fwd(x, w)
    ref = x.reshape(-1, 6).astype(np.float64) @ w.reshape(6, 7).astype(np.float64)
    tol = 1e-13 if dtype == np.float64 else 1e-6
    assert np.abs(y.reshape(-1, 7) - ref).max() <= tol * np.abs(ref).max()


def test_conv3x3_matches_scipy_correlate(oracle):
    x = rnd(2, 6, 5, 3)
    w = rnd(3, 3, 3, 4)
    y = oracle.conv_fwd(x, w)
    ref = np.zeros((2, 6, 5, 4))
    for n in range(2):
        for k in range(4):
            for c in range(3):
                ref[n, :, :, k] += correlate2d(x[n, :, :, c], w[:, :, c, k], mode="same")
    assert np.abs(y - ref).max() < 1e-12


def test_conv3x3_delta_filter_is_identity(oracle):
    x = rnd(2, 5, 6, 4)
    w = np.zeros((3, 3, 4, 4))
    w[1, 1] = np.eye(4)
    assert np.array_equal(oracle.conv_fwd(x, w), x)
    # a delta at tap (0,0) shifts the image down/right by one with zero fill (pad = 1)
    w = np.zeros((3, 3, 4, 4))
    w[0, 0] = np.eye(4)
    y = oracle.conv_fwd(x, w)
    assert np.array_equal(y[:, 1:, 1:], x[:, :-1, :-1])
    assert np.all(y[:, 0] == 0) and np.all(y[:, :, 0] == 0)


@pytest.mark.parametrize("R", [1, 3])
def test_stride2_is_subsampled_stride1(oracle, R):
    x = rnd(2, 8, 6, 3)
    w = rnd(R, R, 3, 5)
    y1 = oracle.conv_fwd(x, w, 1)
    y2 = oracle.conv_fwd(x, w, 2)
    assert y2.shape == (2, 4, 3, 5)
    assert np.array_equal(y2, y1[:, ::2, ::2])


# ------------------------------------------------------------------ adjoints
@pytest.mark.parametrize("R,stride,h,w", [(1, 1, 4, 5), (3, 1, 5, 4), (3, 2, 6, 8), (1, 2, 4, 6)])
def test_dgrad_wgrad_are_adjoints(oracle, R, stride, h, w):
    x = rnd(3, h, w, 4)
    wt = rnd(R, R, 4, 5)
    y = oracle.conv_fwd(x, wt, stride)
    dy = rnd(*y.shape)
    lhs = np.sum(y * dy)
    dx = oracle.conv_dgrad(dy, wt, (h, w), stride)
    dw = oracle.conv_wgrad(x, dy, R, stride)
    assert dx.shape == x.shape and dw.shape == wt.shape
    assert abs(lhs - np.sum(x * dx)) <= 1e-12 * abs(lhs)
    assert abs(lhs - np.sum(wt * dw)) <= 1e-12 * abs(lhs)


def test_wgrad_accumulates(oracle):
    x, dy = rnd(2, 4, 4, 3), rnd(2, 4, 4, 2)
    dw1 = oracle.conv_wgrad(x, dy, 3)
    import ctypes as C
    dw = dw1.copy()
    oracle.lib().oracle_conv_wgrad_f64(x.ctypes.data_as(C.c_void_p), dy.ctypes.data_as(C.c_void_p),
                                       dw.ctypes.data_as(C.c_void_p), 2, 4, 4, 3, 2, 3, 1)
    assert np.allclose(dw, 2 * dw1, rtol=1e-14)


# ------------------------------------------------------------------ Eq. 1-7
def test_two_linear_partitions_closed_form(oracle):
    """Eq. 3-7 with 1x1 convolutions as the two weights: V = X W1, Y' = V W2, G = dL/dY'.
    partial_error = G W2^T, D1 = X^T partial_error, D2 = V^T G."""
    X, W1, W2 = rnd(2, 3, 3, 4), rnd(1, 1, 4, 5), rnd(1, 1, 5, 3)
    V = oracle.conv_fwd(X, W1)
    Y = oracle.conv_fwd(V, W2)
    G = rnd(*Y.shape)
    perr = oracle.conv_dgrad(G, W2, (3, 3))
    D2 = oracle.conv_wgrad(V, G, 1)
    D1 = oracle.conv_wgrad(X, perr, 1)
    Xm, Gm = X.reshape(-1, 4), G.reshape(-1, 3)
    w1, w2 = W1.reshape(4, 5), W2.reshape(5, 3)
    assert np.allclose(perr.reshape(-1, 5), Gm @ w2.T, rtol=1e-13, atol=1e-13)
    assert np.allclose(D2.reshape(5, 3), (Xm @ w1).T @ Gm, rtol=1e-13, atol=1e-13)
    assert np.allclose(D1.reshape(4, 5), Xm.T @ (Gm @ w2.T), rtol=1e-13, atol=1e-13)


def test_two_linear_partitions_worked_fixture(oracle):
    """Hand-worked numbers for Eq. 3-7 (tests/golden/eq1_7_two_layer.txt)."""
    path = os.path.join(os.path.dirname(__file__), "golden", "eq1_7_two_layer.txt")
    vals = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = np.array([float(t) for t in v.split()])
    X = vals["X"].reshape(1, 1, 2, 2)         # two pixels, two channels
    W1 = vals["W1"].reshape(1, 1, 2, 2)
    W2 = vals["W2"].reshape(1, 1, 2, 1)
    G = vals["G"].reshape(1, 1, 2, 1)
    V = oracle.conv_fwd(X, W1)
    assert np.array_equal(V.ravel(), vals["V"])
    assert np.array_equal(oracle.conv_fwd(V, W2).ravel(), vals["Y"])
    perr = oracle.conv_dgrad(G, W2, (1, 2))
    assert np.array_equal(perr.ravel(), vals["partial_error"])
    assert np.array_equal(oracle.conv_wgrad(X, perr, 1).ravel(), vals["D1"])
    assert np.array_equal(oracle.conv_wgrad(V, G, 1).ravel(), vals["D2"])


# ------------------------------------------------------------------ BN + ReLU
def test_bn_forward_moments_and_library_formula(oracle):
    x = rnd(4, 5, 3, 6) * 3.0 + 1.5
    gamma, beta = rng.uniform(0.5, 1.5, 6), rnd(6) * 0.3
    eps = 1e-5
    a, mean, invstd = oracle.bn_relu_fwd(x, gamma, beta, eps)
    xm = x.reshape(-1, 6)
    assert np.allclose(mean, xm.mean(0), rtol=1e-13)
    assert np.allclose(invstd, 1 / np.sqrt(xm.var(0) + eps), rtol=1e-13)
    xh = (xm - mean) * invstd
    assert np.abs(xh.mean(0)).max() < 1e-13
    assert np.allclose((xh ** 2).mean(0), xm.var(0) / (xm.var(0) + eps), rtol=1e-12)
    assert np.allclose(a.reshape(-1, 6), np.maximum(gamma * xh + beta, 0), atol=1e-13)
    # gamma = 1, beta = 0: output is relu(xhat)
    a1, _, _ = oracle.bn_relu_fwd(x, np.ones(6), np.zeros(6), eps)
    assert np.allclose(a1.reshape(-1, 6), np.maximum(xh, 0), atol=1e-13)


def test_bn_frozen_mode_is_per_sample_affine(oracle):
    x = rnd(3, 2, 2, 4)
    gamma, beta = rng.uniform(0.5, 1.5, 4), rnd(4)
    a, mean, invstd = oracle.bn_relu_fwd(x, gamma, beta, 1e-5, mode=1)
    assert np.all(mean == 0) and np.allclose(invstd, 1 / np.sqrt(1 + 1e-5))
    assert np.allclose(a, np.maximum(gamma * x / np.sqrt(1 + 1e-5) + beta, 0), atol=1e-14)


def test_bn_backward_identities(oracle):
    x = rnd(4, 3, 3, 5) * 2 + 0.7
    gamma, beta = rng.uniform(0.5, 1.5, 5), rnd(5) * 0.3
    a, mean, invstd = oracle.bn_relu_fwd(x, gamma, beta)
    da = rnd(*x.shape)
    dx, dg, db = oracle.bn_relu_bwd(x, da, gamma, beta, mean, invstd)
    xh = (x.reshape(-1, 5) - mean) * invstd
    dz = da.reshape(-1, 5) * (a.reshape(-1, 5) > 0)
    assert np.allclose(db, dz.sum(0), rtol=1e-12)
    assert np.allclose(dg, (dz * xh).sum(0), rtol=1e-12)
    dxm = dx.reshape(-1, 5)
    scale = np.abs(dxm).max()
    assert np.abs(dxm.sum(0)).max() < 1e-12 * scale * len(dxm)
    # sum dx*xhat = gamma*invstd*dgamma*(1 - mean(xhat^2)) = gamma*invstd^3*eps*dgamma (zero as eps -> 0)
    assert np.allclose((dxm * xh).sum(0), gamma * invstd ** 3 * 1e-5 * dg, rtol=1e-6,
                       atol=1e-12 * scale * len(dxm))


def test_bn_backward_finite_difference(oracle):
    x = rnd(3, 2, 2, 3) * 1.3 + 0.4
    gamma, beta = rng.uniform(0.5, 1.5, 3), rnd(3) * 0.3
    da = rnd(*x.shape)

    def f(xx, g, b):
        return np.sum(oracle.bn_relu_fwd(xx, g, b)[0] * da)

    a, mean, invstd = oracle.bn_relu_fwd(x, gamma, beta)
    dx, dg, db = oracle.bn_relu_bwd(x, da, gamma, beta, mean, invstd)
    h = 1e-6
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        assert abs((f(xp, gamma, beta) - f(xm, gamma, beta)) / (2 * h) - dx[idx]) < 1e-6
    for c in range(3):
        e = np.zeros(3)
        e[c] = h
        assert abs((f(x, gamma + e, beta) - f(x, gamma - e, beta)) / (2 * h) - dg[c]) < 1e-6
        assert abs((f(x, gamma, beta + e) - f(x, gamma, beta - e)) / (2 * h) - db[c]) < 1e-6


# ------------------------------------------------------------------ head
def test_softmax_ce_closed_forms(oracle):
    n, C, classes = 5, 4, 10
    a = np.abs(rnd(n, 2, 3, C))
    labels = rng.integers(0, classes, n)
    # zero weights and bias -> zero logits -> loss = ln(classes) per sample
    loss, g, dl = oracle.head_fwd(a, np.zeros((C, classes)), np.zeros(classes), labels, divisor=n)
    assert abs(loss - np.log(10.0)) < 1e-14 and abs(np.log(10.0) - 2.302585092994046) < 1e-15
    assert np.allclose(g, a.mean((1, 2)), rtol=1e-14)
    assert np.allclose(dl.sum(1), 0, atol=1e-16)
    loss1000, _, _ = oracle.head_fwd(a, np.zeros((C, 1000)), np.zeros(1000), labels, divisor=n)
    assert abs(loss1000 - 6.907755278982137) < 1e-13
    # general logits: against scipy's logsumexp
    from scipy.special import logsumexp, softmax
    wfc, bfc = rnd(C, classes), rnd(classes)
    B = 20                                           # divisor = full batch, larger than this micro-batch
    loss, g, dl = oracle.head_fwd(a, wfc, bfc, labels, divisor=B)
    logits = a.mean((1, 2)) @ wfc + bfc
    ref = np.sum(logsumexp(logits, axis=1) - logits[np.arange(n), labels]) / B
    assert abs(loss - ref) < 1e-13
    p = softmax(logits, axis=1)
    assert np.allclose(dl.sum(1), 0, atol=1e-15)
    assert abs(dl[np.arange(n), labels].sum() - (p[np.arange(n), labels].sum() - n) / B) < 1e-14
    # huge logits must not overflow (max-subtraction)
    loss_big, _, _ = oracle.head_fwd(a, wfc * 1e4, bfc, labels, divisor=B)
    assert np.isfinite(loss_big)


def test_head_backward_finite_difference(oracle):
    n, C, classes = 3, 4, 5
    a = np.abs(rnd(n, 2, 2, C))
    wfc, bfc = rnd(C, classes), rnd(classes)
    labels = rng.integers(0, classes, n)
    _, g, dl = oracle.head_fwd(a, wfc, bfc, labels, divisor=7)
    dwfc, dbfc, da = oracle.head_bwd(g, dl, wfc, (2, 2))
    f = lambda aa, w, b: oracle.head_fwd(aa, w, b, labels, divisor=7)[0]
    h = 1e-6
    for idx in np.ndindex(*wfc.shape):
        e = np.zeros_like(wfc)
        e[idx] = h
        assert abs((f(a, wfc + e, bfc) - f(a, wfc - e, bfc)) / (2 * h) - dwfc[idx]) < 1e-8
    for j in range(classes):
        e = np.zeros(classes)
        e[j] = h
        assert abs((f(a, wfc, bfc + e) - f(a, wfc, bfc - e)) / (2 * h) - dbfc[j]) < 1e-8
    for idx in np.ndindex(*a.shape):
        e = np.zeros_like(a)
        e[idx] = h
        assert abs((f(a + e, wfc, bfc) - f(a - e, wfc, bfc)) / (2 * h) - da[idx]) < 1e-8


# ------------------------------------------------------------------ bf16 storage reading
def test_bf16_rounding_matches_library_and_closed_forms(oracle):
    import torch
    vals = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-6, 6, 2000),
                           [0.0, -0.0, 1.0, -1.0, 3.0e38, 1e-40]]).astype(np.float32)
    got = np.array([oracle.round_bf16(v) for v in vals], np.float32)
    ref = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got, ref)
    # 8 significant bits, ties to even: 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> 1 (even mantissa)
    assert oracle.round_bf16(1.0 + 2.0 ** -8) == 1.0
    assert oracle.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert oracle.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert oracle.round_bf16(257.0) == 256.0 and oracle.round_bf16(259.0) == 260.0


def test_bf16_storage_rounds_outputs_once_and_is_exact_on_representable_data(oracle):
    x = rng.integers(-3, 4, (2, 4, 4, 3)).astype(np.float32)
    w = rng.integers(-2, 3, (3, 3, 3, 2)).astype(np.float32)
    add = rng.integers(-5, 6, (2, 4, 4, 2)).astype(np.float32)
    # small integers: every product, sum and result is representable -> both readings agree exactly
    assert np.array_equal(oracle.conv_fwd(x, w, add=add, storage="bf16"), oracle.conv_fwd(x, w) + add)
    # weights are used as bfloat16, the sum with the shortcut is rounded once
    x1 = np.ones((1, 1, 1, 1), np.float32)
    w1 = np.full((1, 1, 1, 1), 1.0 + 2.0 ** -9, np.float32)          # rounds to 1.0 as an operand
    a1 = np.full((1, 1, 1, 1), 2.0 ** -8, np.float32)
    y = oracle.conv_fwd(x1, w1, add=a1, storage="bf16")
    assert y.item() == oracle.round_bf16(1.0 + 2.0 ** -8) == 1.0      # rnd(1*1 + 2^-8), not rnd(1) + 2^-8
    assert oracle.conv_fwd(x1, w1, add=a1).item() == np.float32(1.0 + 2.0 ** -9 + 2.0 ** -8)
    dx = oracle.conv_dgrad(x1, w1, (1, 1), storage="bf16")
    assert dx.item() == 1.0
    # BN+ReLU output and backward output are stored values
    xb = rng.standard_normal((16, 8)).astype(np.float32)
    g, b = np.ones(8, np.float32), np.zeros(8, np.float32)
    a, mean, inv = oracle.bn_relu_fwd(xb, g, b, storage="bf16")
    a0, _, _ = oracle.bn_relu_fwd(xb, g, b)
    import torch
    assert np.array_equal(a, torch.from_numpy(a0).to(torch.bfloat16).float().numpy())
    da = rng.standard_normal((16, 8)).astype(np.float32)
    sk = rng.standard_normal((16, 8)).astype(np.float32)
    d1, dg1, db1 = oracle.bn_relu_bwd(xb, da, g, b, mean, inv, skip=sk, storage="bf16")
    d0, dg0, db0 = oracle.bn_relu_bwd(xb, da, g, b, mean, inv)
    assert np.array_equal(dg1, dg0) and np.array_equal(db1, db0)     # reductions are not rounded
    assert np.array_equal(d1, torch.from_numpy((d0.astype(np.float64) + sk).astype(np.float32)).to(torch.bfloat16).float().numpy())
