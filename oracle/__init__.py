"""CPU oracle -- TEST INFRASTRUCTURE, not the product.

ctypes wrapper around liboracle.so (oracle/oracle.cpp): a plain direct-loop CPU
implementation of one model partition's forward / backward / gradient
accumulation / SGD step, written from the paper's description of the method
(distributed back-propagation with partial errors, Eq. 1-7; micro-batch
pipelining; one synchronous update per batch).  Only tests, the smoke check and
the benchmark's cpu_baseline leg may import this package; it shares no code
with the HIP path and never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile liboracle.so with g++ (OpenMP) if it is missing or older than its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        L = _lib
        L.oracle_partition_create.restype = C.c_void_p
        L.oracle_partition_create.argtypes = [C.c_void_p, C.c_double, C.c_void_p, C.c_void_p, C.c_int]
        L.oracle_partition_destroy.argtypes = [C.c_void_p]
        L.oracle_partition_destroy.restype = None
        L.oracle_n_params.restype = C.c_size_t
        L.oracle_n_params.argtypes = [C.c_void_p]
        L.oracle_forward_microbatch.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_backward_microbatch.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.oracle_forward_microbatch_cut.argtypes = [C.c_void_p, C.c_int] + [C.c_void_p] * 6
        L.oracle_backward_microbatch_cut.argtypes = [C.c_void_p, C.c_int] + [C.c_void_p] * 4
        L.oracle_grad_accum_read.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        L.oracle_forward_inference.argtypes = [C.c_void_p] * 5
        L.oracle_set_bn_momentum.argtypes = [C.c_void_p, C.c_double]
        L.oracle_set_bn_momentum.restype = None
        L.oracle_n_bn_running.argtypes = [C.c_void_p]
        L.oracle_n_bn_running.restype = C.c_size_t
        L.oracle_bn_running_read.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        L.oracle_bn_running_write.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        L.oracle_grad_accum_zero.argtypes = [C.c_void_p]
        L.oracle_sgd_step.argtypes = [C.c_void_p, C.c_double, C.c_double]
        L.oracle_params_read.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        L.oracle_params_write.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        L.oracle_round_bf16.argtypes = [C.c_float]
        L.oracle_round_bf16.restype = C.c_float
        for suf in ("f32", "f64"):
            i, d, p, z = C.c_int, C.c_double, C.c_void_p, C.c_size_t
            getattr(L, f"oracle_conv_fwd_{suf}").argtypes = [p, p, p, i, i, i, i, i, i, i, p, i]
            getattr(L, f"oracle_conv_dgrad_{suf}").argtypes = [p, p, p, i, i, i, i, i, i, i, p, i]
            getattr(L, f"oracle_conv_wgrad_{suf}").argtypes = [p, p, p, i, i, i, i, i, i, i]
            getattr(L, f"oracle_bn_relu_fwd_{suf}").argtypes = [p, p, p, p, p, p, z, i, d, i, i]
            getattr(L, f"oracle_bn_relu_bwd_{suf}").argtypes = [p, p, p, p, p, p, p, p, p, z, i, i, p, i]
            getattr(L, f"oracle_head_fwd_{suf}").argtypes = [p, p, p, p, p, p, i, i, i, i, d]
            getattr(L, f"oracle_head_fwd_{suf}").restype = d
            getattr(L, f"oracle_head_bwd_{suf}").argtypes = [p, p, p, p, p, p, i, i, i, i]
            getattr(L, f"oracle_bias_act_fwd_{suf}").argtypes = [p, p, p, z, i, i]
            getattr(L, f"oracle_bias_act_bwd_{suf}").argtypes = [p, p, p, p, z, i, i]
            getattr(L, f"oracle_maxpool2_fwd_{suf}").argtypes = [p, p, i, i, i, i]
            getattr(L, f"oracle_maxpool2_bwd_{suf}").argtypes = [p, p, p, i, i, i, i]
            getattr(L, f"oracle_bn_add_relu_fwd_{suf}").argtypes = [p, p, p, p, p, p, p, z, i, d, i]
            getattr(L, f"oracle_bn_add_relu_bwd_{suf}").argtypes = [p, p, p, p, p, p, p, p, p, p, z, i, i]
            for nm in ("conv_fwd", "conv_dgrad", "conv_wgrad", "bn_relu_fwd", "bn_relu_bwd", "head_bwd", "bias_act_fwd",
                       "bias_act_bwd", "maxpool2_fwd", "maxpool2_bwd", "bn_add_relu_fwd", "bn_add_relu_bwd"):
                getattr(L, f"oracle_{nm}_{suf}").restype = None
    return _lib


def _suf(dtype):
    return "f64" if np.dtype(dtype) == np.float64 else "f32"


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


# ---------------------------------------------------------------------------
# single operations (NHWC activations, [R][S][Cin][Cout] weights)
# ---------------------------------------------------------------------------
def conv_out_hw(h, w, R, stride):
    pad = (R - 1) // 2
    return (h + 2 * pad - R) // stride + 1, (w + 2 * pad - R) // stride + 1


STORAGE = {"none": 0, "bf16": 1}


def round_bf16(v: float) -> float:
    """Nearest-even bfloat16 of a float32 value (the oracle's storage rounding)."""
    return float(lib().oracle_round_bf16(float(v)))


def conv_fwd(x, w, stride=1, add=None, storage="none"):
    dt = x.dtype
    x, w = _c(x, dt), _c(w, dt)
    n, h, wd, cin = x.shape
    R, _, _, cout = w.shape
    ho, wo = conv_out_hw(h, wd, R, stride)
    y = np.empty((n, ho, wo, cout), dt)
    add = _c(add, dt) if add is not None else None
    getattr(lib(), f"oracle_conv_fwd_{_suf(dt)}")(_p(x), _p(w), _p(y), n, h, wd, cin, cout, R, stride,
                                                  _p(add), STORAGE[storage])
    return y


def conv_dgrad(dy, w, in_hw, stride=1, add=None, storage="none"):
    dt = dy.dtype
    dy, w = _c(dy, dt), _c(w, dt)
    n = dy.shape[0]
    R, _, cin, cout = w.shape
    h, wd = in_hw
    dx = np.empty((n, h, wd, cin), dt)
    add = _c(add, dt) if add is not None else None
    getattr(lib(), f"oracle_conv_dgrad_{_suf(dt)}")(_p(dy), _p(w), _p(dx), n, h, wd, cin, cout, R, stride,
                                                    _p(add), STORAGE[storage])
    return dx


def conv_wgrad(x, dy, R, stride=1):
    dt = x.dtype
    x, dy = _c(x, dt), _c(dy, dt)
    n, h, wd, cin = x.shape
    cout = dy.shape[-1]
    dw = np.zeros((R, R, cin, cout), np.float64)
    getattr(lib(), f"oracle_conv_wgrad_{_suf(dt)}")(_p(x), _p(dy), _p(dw), n, h, wd, cin, cout, R, stride)
    return dw


def bn_relu_fwd(x, gamma, beta, eps=1e-5, mode=0, storage="none"):
    dt = x.dtype
    x, gamma, beta = _c(x, dt), _c(gamma, dt), _c(beta, dt)
    Cc = x.shape[-1]
    M = x.size // Cc
    a = np.empty_like(x)
    mean, invstd = np.empty(Cc), np.empty(Cc)
    getattr(lib(), f"oracle_bn_relu_fwd_{_suf(dt)}")(_p(x), _p(gamma), _p(beta), _p(a), _p(mean), _p(invstd),
                                                     M, Cc, eps, mode, STORAGE[storage])
    return a, mean, invstd


def bn_relu_bwd(x, da, gamma, beta, mean, invstd, mode=0, skip=None, storage="none"):
    dt = x.dtype
    x, da, gamma, beta = _c(x, dt), _c(da, dt), _c(gamma, dt), _c(beta, dt)
    mean, invstd = _c(mean, np.float64), _c(invstd, np.float64)
    Cc = x.shape[-1]
    M = x.size // Cc
    dx = np.empty_like(x)
    dg, db = np.zeros(Cc), np.zeros(Cc)
    skip = _c(skip, dt) if skip is not None else None
    getattr(lib(), f"oracle_bn_relu_bwd_{_suf(dt)}")(_p(x), _p(da), _p(gamma), _p(beta), _p(mean), _p(invstd),
                                                     _p(dx), _p(dg), _p(db), M, Cc, mode, _p(skip), STORAGE[storage])
    return dx, dg, db


def head_fwd(a, wfc, bfc, labels, divisor):
    dt = a.dtype
    a, wfc, bfc = _c(a, dt), _c(wfc, dt), _c(bfc, dt)
    labels = _c(labels, np.int32)
    n, h, w, Cc = a.shape
    classes = wfc.shape[1]
    g = np.empty((n, Cc), dt)
    dl = np.empty((n, classes), dt)
    loss = getattr(lib(), f"oracle_head_fwd_{_suf(dt)}")(_p(a), _p(wfc), _p(bfc), _p(labels), _p(g), _p(dl),
                                                         n, h * w, Cc, classes, float(divisor))
    return loss, g, dl


def head_bwd(g, dlogits, wfc, hw):
    dt = g.dtype
    g, dlogits, wfc = _c(g, dt), _c(dlogits, dt), _c(wfc, dt)
    n, Cc = g.shape
    classes = wfc.shape[1]
    h, w = hw
    dwfc, dbfc = np.zeros((Cc, classes)), np.zeros(classes)
    da = np.empty((n, h, w, Cc), dt)
    getattr(lib(), f"oracle_head_bwd_{_suf(dt)}")(_p(g), _p(dlogits), _p(wfc), _p(dwfc), _p(dbfc), _p(da),
                                                  n, h * w, Cc, classes)
    return dwfc, dbfc, da


def bias_act_fwd(x, bias, relu=True):
    """y = x + bias[c], then max(., 0) if relu."""
    dt = x.dtype
    x, bias = _c(x, dt), _c(bias, dt)
    Cc = x.shape[-1]
    y = np.empty_like(x)
    getattr(lib(), f"oracle_bias_act_fwd_{_suf(dt)}")(_p(x), _p(bias), _p(y), x.size // Cc, Cc, int(relu))
    return y


def bias_act_bwd(y, dy, relu=True):
    """Returns dx = dy*[y>0] (or dy) and dbias = sum over rows of dx."""
    dt = y.dtype
    y, dy = _c(y, dt), _c(dy, dt)
    Cc = y.shape[-1]
    dx, db = np.empty_like(y), np.zeros(Cc)
    getattr(lib(), f"oracle_bias_act_bwd_{_suf(dt)}")(_p(y), _p(dy), _p(dx), _p(db), y.size // Cc, Cc, int(relu))
    return dx, db


def maxpool2_fwd(x):
    dt = x.dtype
    x = _c(x, dt)
    n, h, w, Cc = x.shape
    y = np.empty((n, h // 2, w // 2, Cc), dt)
    getattr(lib(), f"oracle_maxpool2_fwd_{_suf(dt)}")(_p(x), _p(y), n, h, w, Cc)
    return y


def maxpool2_bwd(x, dy):
    dt = x.dtype
    x, dy = _c(x, dt), _c(dy, dt)
    n, h, w, Cc = x.shape
    dx = np.empty_like(x)
    getattr(lib(), f"oracle_maxpool2_bwd_{_suf(dt)}")(_p(x), _p(dy), _p(dx), n, h, w, Cc)
    return dx


def bn_add_relu_fwd(x, gamma, beta, add, eps=1e-5, mode=0):
    """y = relu(bn(x) + add); returns y, mean, invstd."""
    dt = x.dtype
    x, gamma, beta, add = _c(x, dt), _c(gamma, dt), _c(beta, dt), _c(add, dt)
    Cc = x.shape[-1]
    y = np.empty_like(x)
    mean, invstd = np.empty(Cc), np.empty(Cc)
    getattr(lib(), f"oracle_bn_add_relu_fwd_{_suf(dt)}")(_p(x), _p(gamma), _p(beta), _p(add), _p(y), _p(mean), _p(invstd),
                                                         x.size // Cc, Cc, eps, mode)
    return y, mean, invstd


def bn_add_relu_bwd(x, y, dy, gamma, mean, invstd, mode=0):
    """Returns dx (through the BatchNorm), dadd = dy*[y>0], dgamma, dbeta."""
    dt = x.dtype
    x, y, dy, gamma = _c(x, dt), _c(y, dt), _c(dy, dt), _c(gamma, dt)
    mean, invstd = _c(mean, np.float64), _c(invstd, np.float64)
    Cc = x.shape[-1]
    dx, dadd = np.empty_like(x), np.empty_like(x)
    dg, db = np.zeros(Cc), np.zeros(Cc)
    getattr(lib(), f"oracle_bn_add_relu_bwd_{_suf(dt)}")(_p(x), _p(y), _p(dy), _p(gamma), _p(mean), _p(invstd), _p(dx), _p(dadd),
                                                         _p(dg), _p(db), x.size // Cc, Cc, mode)
    return dx, dadd, dg, db


# ---------------------------------------------------------------------------
# the partition
# ---------------------------------------------------------------------------
class OraclePartition:
    """Host-pointer twin of the HIP library's partition handle.  `spec` is any object with
    the fields of workloads.PartitionSpec (duck-typed; this package imports nothing else)."""

    def __init__(self, spec, params, dtype=np.float32, storage="none"):
        self.spec = spec
        self.dtype = np.dtype(dtype)
        blocks = np.array([[b.kind, b.c_in, b.c_mid, b.c_out, b.stride] for b in spec.blocks],
                          dtype=np.int32).reshape(-1, 5)
        desc = np.array([spec.in_h, spec.in_w, spec.in_c, int(spec.has_stem), spec.stem_c_out,
                         len(spec.blocks), int(spec.has_head), spec.num_classes, spec.microbatch,
                         spec.num_microbatches, spec.divisor, spec.bn_mode, STORAGE[storage],
                         getattr(spec, "first_from", 0), getattr(spec, "last_to", 0),
                         int(getattr(spec, "head_bn", True))], dtype=np.int32)
        params = _c(params, self.dtype)
        self._h = lib().oracle_partition_create(_p(desc), float(spec.bn_eps), _p(blocks), _p(params),
                                                int(self.dtype == np.float64))
        if not self._h:
            raise ValueError("oracle: invalid partition description")
        self.n_params = lib().oracle_n_params(self._h)
        if self.n_params != params.size:
            raise ValueError(f"oracle: expected {self.n_params} parameters, got {params.size}")
        oh, ow, oc = spec.out_shape()
        self.out_shape = (spec.microbatch, oh, ow, oc)
        self.in_shape = (spec.microbatch, spec.in_h, spec.in_w, spec.in_c)
        self.skip_in_shape = (spec.microbatch,) + tuple(spec.skip_in_shape()) if getattr(spec, "has_skip_in", False) else None
        self.skip_out_shape = (spec.microbatch,) + tuple(spec.skip_out_shape()) if getattr(spec, "has_skip_out", False) else None
        self.loss = np.zeros(1, np.float64)

    def close(self):
        if self._h:
            lib().oracle_partition_destroy(self._h)
            self._h = None

    __del__ = close

    @staticmethod
    def _check(rc, what):
        if rc != 0:
            raise RuntimeError(f"oracle {what}: status {rc}")

    def forward(self, mb, act_in, labels=None, skip_in=None):
        """Returns act_out, or (act_out, skip_out) when the last block is cut before its end."""
        act_in = _c(act_in, self.dtype)
        assert act_in.shape == self.in_shape, (act_in.shape, self.in_shape)
        out = None if self.spec.has_head else np.empty(self.out_shape, self.dtype)
        lab = _c(labels, np.int32) if labels is not None else None
        sk = _c(skip_in, self.dtype) if skip_in is not None else None
        assert (sk is None) == (self.skip_in_shape is None) and (sk is None or sk.shape == self.skip_in_shape)
        sko = np.empty(self.skip_out_shape, self.dtype) if self.skip_out_shape else None
        self._check(lib().oracle_forward_microbatch_cut(self._h, mb, _p(act_in), _p(sk), _p(lab), _p(out), _p(sko),
                                                        _p(self.loss)), "forward")
        return (out, sko) if sko is not None else out

    def backward(self, mb, err_in=None, want_err_out=True, skip_err_in=None):
        """Returns err_out, or (err_out, skip_err_out) when the first block is cut after its start."""
        e = _c(err_in, self.dtype) if err_in is not None else None
        if e is not None:
            assert e.shape == self.out_shape
        se = _c(skip_err_in, self.dtype) if skip_err_in is not None else None
        assert (se is None) == (self.skip_out_shape is None) and (se is None or se.shape == self.skip_out_shape)
        out = np.empty(self.in_shape, self.dtype) if want_err_out else None
        seo = np.empty(self.skip_in_shape, self.dtype) if self.skip_in_shape else None
        self._check(lib().oracle_backward_microbatch_cut(self._h, mb, _p(e), _p(se), _p(out), _p(seo)), "backward")
        return (out, seo) if seo is not None else out

    def set_bn_momentum(self, momentum):
        """Training forwards move the running statistics: r <- momentum*r + (1-momentum)*batch (1: never)."""
        lib().oracle_set_bn_momentum(self._h, float(momentum))

    def bn_running(self):
        """Running statistics (float64): per BatchNorm in model order mean[c] then variance[c]."""
        r = np.empty(lib().oracle_n_bn_running(self._h), np.float64)
        self._check(lib().oracle_bn_running_read(self._h, _p(r), r.size), "bn_running_read")
        return r

    def set_bn_running(self, r):
        r = _c(r, np.float64)
        self._check(lib().oracle_bn_running_write(self._h, _p(r), r.size), "bn_running_write")

    def infer(self, act_in, skip_in=None):
        """Inference forward (BatchNorm by running statistics): logits [b, classes] with a head, else act_out
        (or (act_out, skip_out))."""
        act_in = _c(act_in, self.dtype)
        assert act_in.shape == self.in_shape
        out = np.empty((self.spec.microbatch, self.spec.num_classes) if self.spec.has_head else self.out_shape, self.dtype)
        sk = _c(skip_in, self.dtype) if skip_in is not None else None
        sko = np.empty(self.skip_out_shape, self.dtype) if self.skip_out_shape else None
        self._check(lib().oracle_forward_inference(self._h, _p(act_in), _p(sk), _p(out), _p(sko)), "forward_inference")
        return (out, sko) if sko is not None else out

    def grad(self):
        g = np.empty(self.n_params, self.dtype)
        self._check(lib().oracle_grad_accum_read(self._h, _p(g), g.size), "grad_accum_read")
        return g

    def zero_grad(self):
        self._check(lib().oracle_grad_accum_zero(self._h), "grad_accum_zero")
        self.loss[:] = 0

    def sgd_step(self, lr, momentum):
        self._check(lib().oracle_sgd_step(self._h, lr, momentum), "sgd_step")
        self.loss[:] = 0

    def params(self):
        p = np.empty(self.n_params, self.dtype)
        self._check(lib().oracle_params_read(self._h, _p(p), p.size), "params_read")
        return p

    def set_params(self, p):
        p = _c(p, self.dtype)
        self._check(lib().oracle_params_write(self._h, _p(p), p.size), "params_write")


def run_step(spec, inputs, dtype=np.float32, sgd=None, storage="none"):
    """One batch: m forwards then m backwards (micro-batch index order).  Returns a dict with
    per-micro-batch act_out / err_out, the loss, the accumulated gradient and, when `sgd` =
    (lr, momentum) is given, the parameters after the step."""
    part = OraclePartition(spec, inputs.params, dtype, storage)
    outs, errs, skip_outs, skip_errs = [], [], [], []
    skip_in = getattr(inputs, "skip_in", None)
    skip_err_in = getattr(inputs, "skip_err_in", None)
    for i in range(spec.num_microbatches):
        o = part.forward(i, inputs.act_in[i], inputs.labels[i] if inputs.labels else None,
                         skip_in[i] if skip_in else None)
        if isinstance(o, tuple):
            skip_outs.append(o[1]); o = o[0]
        outs.append(o)
    loss = float(part.loss[0])
    for i in range(spec.num_microbatches):
        e = part.backward(i, inputs.err_in[i] if inputs.err_in else None, want_err_out=not spec.has_stem,
                          skip_err_in=skip_err_in[i] if skip_err_in else None)
        if isinstance(e, tuple):
            skip_errs.append(e[1]); e = e[0]
        errs.append(e)
    res = {"act_out": outs, "err_out": errs, "loss": loss, "grad": part.grad()}
    if skip_outs:
        res["skip_out"] = skip_outs
    if skip_errs:
        res["skip_err_out"] = skip_errs
    if sgd is not None:
        part.sgd_step(*sgd)
        res["params"] = part.params()
    part.close()
    return res
