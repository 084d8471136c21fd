"""ctypes binding to libhpf.so -- argument marshalling only.

Functions carry the names of the C ABI (include/hpf.h) and take raw device addresses
(ints, e.g. torch.Tensor.data_ptr()) and stream handles; every step of the path runs in
the library's HIP kernels.  `Partition` is a small convenience wrapper that owns the torch
arena tensor and checks shapes/dtypes.  There is no CPU fallback: if the library cannot be
loaded the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhpf.so")

HPF_ABI_VERSION = 2
HPF_OK, HPF_EINVAL, HPF_ESTATE, HPF_ENOMEM, HPF_EDEVICE, HPF_EUNSUPPORTED = range(6)
HPF_F32, HPF_BF16 = 0, 1
STATUS_NAMES = {0: "HPF_OK", 1: "HPF_EINVAL", 2: "HPF_ESTATE", 3: "HPF_ENOMEM", 4: "HPF_EDEVICE",
                5: "HPF_EUNSUPPORTED"}


class hpf_block_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("c_in", C.c_int32), ("c_mid", C.c_int32), ("c_out", C.c_int32),
                ("stride", C.c_int32)]


class hpf_partition_desc(C.Structure):
    _fields_ = [("abi_version", C.c_uint32), ("in_h", C.c_int32), ("in_w", C.c_int32), ("in_c", C.c_int32),
                ("has_stem", C.c_int32), ("stem_c_out", C.c_int32), ("n_blocks", C.c_int32),
                ("blocks", C.POINTER(hpf_block_desc)), ("has_head", C.c_int32), ("num_classes", C.c_int32),
                ("microbatch", C.c_int32), ("num_microbatches", C.c_int32), ("loss_divisor", C.c_int32),
                ("compute_dtype", C.c_int), ("bn_eps", C.c_float), ("bn_mode", C.c_int32),
                ("first_block_from_conv", C.c_int32), ("last_block_to_conv", C.c_int32)]


class hpf_sizes(C.Structure):
    _fields_ = [("n_params", C.c_size_t), ("arena_bytes", C.c_size_t), ("stash_bytes", C.c_size_t),
                ("act_in_elems", C.c_size_t), ("act_out_elems", C.c_size_t),
                ("skip_in_elems", C.c_size_t), ("skip_out_elems", C.c_size_t), ("n_bn_running", C.c_size_t)]


class HpfError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1911_05146_amd.build` "
                          "(there is no fallback path)")
    # PyTorch ships its own HIP runtime; whichever runtime is loaded first serves the whole process, and the
    # device tensors handed to this library come from PyTorch's: load it first.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    L.hpf_last_error.restype = C.c_char_p
    L.hpf_partition_sizes.argtypes = [C.POINTER(hpf_partition_desc), C.POINTER(hpf_sizes)]
    L.hpf_partition_create.argtypes = [C.POINTER(hpf_partition_desc), vp, sz, vp, C.POINTER(vp)]
    L.hpf_forward_microbatch.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    L.hpf_backward_microbatch.argtypes = [vp, i32, vp, vp, vp]
    L.hpf_forward_microbatch_cut.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp]
    L.hpf_backward_microbatch_cut.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    L.hpf_forward_microbatches.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp]
    L.hpf_backward_microbatches.argtypes = [vp, i32, i32, vp, vp, vp]
    L.hpf_grad_accum_read.argtypes = [vp, vp, sz, i32, vp]
    L.hpf_grad_accum_zero.argtypes = [vp, vp]
    L.hpf_sgd_step.argtypes = [vp, C.c_float, C.c_float, vp]
    L.hpf_params_read.argtypes = [vp, vp, sz]
    L.hpf_partition_destroy.argtypes = [vp]
    L.hpf_partition_destroy.restype = None
    L.hpf_partition_set_graphs.argtypes = [vp, i32]
    L.hpf_partition_set_fusion.argtypes = [vp, i32]
    L.hpf_partition_set_bn_momentum.argtypes = [vp, C.c_float]
    L.hpf_bn_running_read.argtypes = [vp, vp, sz]
    L.hpf_bn_running_write.argtypes = [vp, vp, sz]
    L.hpf_forward_inference.argtypes = [vp, vp, vp, vp, vp, vp]
    L.hpf_forward_inference_group.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    L.hpf_partition_set_profiling.argtypes = [vp, i32]
    L.hpf_partition_profile_read.argtypes = [vp, vp, i32, vp]
    L.hpf_op_workspace_bytes.argtypes = [i32, i32, i32]
    L.hpf_op_workspace_bytes.restype = sz
    L.hpf_op_conv_forward.argtypes = [C.c_int, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, sz, i32, vp]
    L.hpf_op_conv_dgrad.argtypes = [C.c_int, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, sz, i32, vp]
    L.hpf_op_conv_wgrad.argtypes = [C.c_int, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp]
    L.hpf_op_bn_relu_forward.argtypes = [C.c_int, vp, vp, vp, C.c_float, vp, vp, i32, i32, vp, sz, vp]
    L.hpf_op_bn_relu_backward.argtypes = [C.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, sz, vp]
    L.hpf_op_bn_relu_forward_noalloc.argtypes = [C.c_int, vp, vp, vp, C.c_float, vp, vp, i32, i32, vp]
    L.hpf_partition_check.argtypes = [vp]
    L.hpf_debug_set_invalid.argtypes = [vp, i32]
    L.hpf_stash_read.argtypes = [vp, i32, i32, i32, vp, sz, C.POINTER(sz), C.POINTER(i32)]
    L.hpf_probe_copy.argtypes = [vp, vp, sz, vp]
    L.hpf_probe_mfma_bf16.argtypes = [vp, i32, i32, i32, vp]
    return L


lib = _load()

EXPORTS = ["hpf_partition_sizes", "hpf_partition_create", "hpf_forward_microbatch", "hpf_backward_microbatch",
           "hpf_forward_microbatch_cut", "hpf_backward_microbatch_cut",
           "hpf_forward_microbatches", "hpf_backward_microbatches",
           "hpf_grad_accum_read", "hpf_grad_accum_zero", "hpf_sgd_step", "hpf_params_read",
           "hpf_partition_destroy", "hpf_partition_set_graphs", "hpf_partition_set_fusion",
           "hpf_partition_set_profiling", "hpf_partition_profile_read", "hpf_partition_set_bn_momentum",
           "hpf_bn_running_read", "hpf_bn_running_write", "hpf_forward_inference", "hpf_forward_inference_group",
           "hpf_last_error", "hpf_op_workspace_bytes", "hpf_op_conv_forward",
           "hpf_op_conv_dgrad", "hpf_op_conv_wgrad", "hpf_op_bn_relu_forward", "hpf_op_bn_relu_backward",
           "hpf_stash_read", "hpf_partition_check", "hpf_debug_set_invalid", "hpf_op_bn_relu_forward_noalloc", "hpf_probe_copy", "hpf_probe_mfma_bf16"]


def hpf_last_error() -> str:
    return lib.hpf_last_error().decode()


def _check(status):
    if status != HPF_OK:
        raise HpfError(status, hpf_last_error())


def make_desc(spec, compute_dtype=HPF_BF16):
    """hpf_partition_desc from an object with the fields of workloads.PartitionSpec.
    Returns (desc, keepalive)."""
    n = len(spec.blocks)
    arr = (hpf_block_desc * max(n, 1))()
    for i, b in enumerate(spec.blocks):
        arr[i] = hpf_block_desc(b.kind, b.c_in, b.c_mid, b.c_out, b.stride)
    d = hpf_partition_desc(HPF_ABI_VERSION, spec.in_h, spec.in_w, spec.in_c, int(spec.has_stem), spec.stem_c_out,
                           n, C.cast(arr, C.POINTER(hpf_block_desc)),
                           (1 if getattr(spec, "head_bn", True) else 2) if spec.has_head else 0, spec.num_classes,
                           spec.microbatch, spec.num_microbatches, spec.divisor, compute_dtype,
                           float(spec.bn_eps), spec.bn_mode, getattr(spec, "first_from", 0), getattr(spec, "last_to", 0))
    return d, arr


def hpf_partition_sizes(desc) -> hpf_sizes:
    out = hpf_sizes()
    _check(lib.hpf_partition_sizes(C.byref(desc), C.byref(out)))
    return out


def hpf_partition_create(desc, device_arena: int, arena_bytes: int, host_params) -> int:
    """host_params: contiguous float32 numpy array."""
    h = C.c_void_p()
    _check(lib.hpf_partition_create(C.byref(desc), device_arena, arena_bytes,
                                    host_params.ctypes.data_as(C.c_void_p), C.byref(h)))
    return h.value


def hpf_forward_microbatch(handle, mb, act_in, labels, act_out, loss_accum, stream=0):
    _check(lib.hpf_forward_microbatch(handle, mb, act_in, labels or None, act_out or None, loss_accum or None,
                                      stream or None))


def hpf_backward_microbatch(handle, mb, err_in, err_out, stream=0):
    _check(lib.hpf_backward_microbatch(handle, mb, err_in or None, err_out or None, stream or None))


def hpf_forward_microbatch_cut(handle, mb, act_in, skip_in, labels, act_out, skip_out, loss_accum, stream=0):
    _check(lib.hpf_forward_microbatch_cut(handle, mb, act_in, skip_in or None, labels or None, act_out or None,
                                          skip_out or None, loss_accum or None, stream or None))


def hpf_backward_microbatch_cut(handle, mb, err_in, skip_err_in, err_out, skip_err_out, stream=0):
    _check(lib.hpf_backward_microbatch_cut(handle, mb, err_in or None, skip_err_in or None, err_out or None,
                                           skip_err_out or None, stream or None))


def _ptr_array(ptrs):
    """(host) array of device pointers from a list of ints; None -> NULL array."""
    if ptrs is None:
        return None
    return (C.c_void_p * len(ptrs))(*[p or None for p in ptrs])


def hpf_forward_microbatches(handle, mb_first, act_in, labels, act_out, loss_accum, stream=0):
    """act_in / labels / act_out: lists of device addresses (labels or act_out may be None)."""
    a, l, o = _ptr_array(act_in), _ptr_array(labels), _ptr_array(act_out)
    _check(lib.hpf_forward_microbatches(handle, mb_first, len(act_in), a, l, o, loss_accum or None, stream or None))


def hpf_backward_microbatches(handle, mb_first, count, err_in, err_out, stream=0):
    e, o = _ptr_array(err_in), _ptr_array(err_out)
    _check(lib.hpf_backward_microbatches(handle, mb_first, count, e, o, stream or None))


def hpf_grad_accum_read(handle, dst, n_floats, dst_is_device, stream=0):
    _check(lib.hpf_grad_accum_read(handle, dst, n_floats, int(dst_is_device), stream or None))


def hpf_grad_accum_zero(handle, stream=0):
    _check(lib.hpf_grad_accum_zero(handle, stream or None))


def hpf_sgd_step(handle, lr, momentum, stream=0):
    _check(lib.hpf_sgd_step(handle, lr, momentum, stream or None))


def hpf_params_read(handle, host_dst, n_floats):
    _check(lib.hpf_params_read(handle, host_dst, n_floats))


def hpf_partition_set_graphs(handle, enable):
    _check(lib.hpf_partition_set_graphs(handle, int(enable)))


def hpf_partition_set_fusion(handle, level):
    _check(lib.hpf_partition_set_fusion(handle, int(level)))


def hpf_partition_set_bn_momentum(handle, momentum):
    _check(lib.hpf_partition_set_bn_momentum(handle, float(momentum)))


def hpf_bn_running_read(handle, host_dst, n_floats):
    _check(lib.hpf_bn_running_read(handle, host_dst, n_floats))


def hpf_bn_running_write(handle, host_src, n_floats):
    _check(lib.hpf_bn_running_write(handle, host_src, n_floats))


def hpf_forward_inference_group(handle, act_in, skip_in, out, skip_out, stream=0):
    """Lists of device addresses (skip lists may be None)."""
    _check(lib.hpf_forward_inference_group(handle, len(act_in), _ptr_array(act_in), _ptr_array(skip_in), _ptr_array(out),
                                           _ptr_array(skip_out), stream or None))


def hpf_forward_inference(handle, act_in, skip_in, out, skip_out, stream=0):
    _check(lib.hpf_forward_inference(handle, act_in, skip_in or None, out, skip_out or None, stream or None))


class hpf_profile_entry(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("launches", C.c_int64), ("total_ms", C.c_double),
                ("bytes_per_launch", C.c_double), ("flops_per_launch", C.c_double)]


def hpf_partition_set_profiling(handle, enable):
    _check(lib.hpf_partition_set_profiling(handle, int(bool(enable))))


def hpf_partition_profile_read(handle, capacity=16):
    buf = (hpf_profile_entry * capacity)()
    n = C.c_int32(0)
    _check(lib.hpf_partition_profile_read(handle, buf, capacity, C.byref(n)))
    return [dict(name=buf[i].name.decode(), launches=int(buf[i].launches), total_ms=float(buf[i].total_ms),
                 bytes_per_launch=float(buf[i].bytes_per_launch), flops_per_launch=float(buf[i].flops_per_launch))
            for i in range(n.value)]


# hpf_tensor_id
(HPF_T_X, HPF_T_C1, HPF_T_C2, HPF_T_Y, HPF_T_GY, HPF_T_DC1, HPF_T_DC2, HPF_T_GX, HPF_T_STATS0, HPF_T_STATS1,
 HPF_T_STATS2, HPF_T_A0, HPF_T_A1, HPF_T_A2, HPF_T_Y0, HPF_T_SC) = range(16)
STASH_WHERE = {1: "act_in", 2: "act_out", 3: "err_in", 4: "err_out", 5: "skip_in", 6: "skip_out", 7: "skip_err_in",
               8: "skip_err_out"}


def hpf_stash_read(handle, mb, unit, tensor, host_dst, nbytes):
    """Returns (where, bytes_needed); where == 0: copied into host_dst."""
    need, where = C.c_size_t(0), C.c_int32(-1)
    _check(lib.hpf_stash_read(handle, mb, unit, tensor, host_dst, nbytes, C.byref(need), C.byref(where)))
    return where.value, need.value


def hpf_partition_check(handle):
    _check(lib.hpf_partition_check(handle))


def hpf_debug_set_invalid(handle, value):
    _check(lib.hpf_debug_set_invalid(handle, int(value)))


def hpf_partition_destroy(handle):
    lib.hpf_partition_destroy(handle)


def hpf_op_workspace_bytes(cin, cout, R) -> int:
    return int(lib.hpf_op_workspace_bytes(cin, cout, R))


def hpf_op_conv_forward(dtype, x, w, y, add, b, h, wd, cin, cout, R, stride, workspace, workspace_bytes,
                        repack=1, stream=0):
    _check(lib.hpf_op_conv_forward(dtype, x, w, y, add or None, b, h, wd, cin, cout, R, stride, workspace,
                                   workspace_bytes, repack, stream or None))


def hpf_op_conv_dgrad(dtype, dy, w, dx, add, b, h, wd, cin, cout, R, stride, workspace, workspace_bytes,
                      repack=1, stream=0):
    _check(lib.hpf_op_conv_dgrad(dtype, dy, w, dx, add or None, b, h, wd, cin, cout, R, stride, workspace,
                                 workspace_bytes, repack, stream or None))


def hpf_op_conv_wgrad(dtype, x, dy, dw, b, h, wd, cin, cout, R, stride, stream=0):
    _check(lib.hpf_op_conv_wgrad(dtype, x, dy, dw, b, h, wd, cin, cout, R, stride, stream or None))


def hpf_op_bn_relu_forward(dtype, x, gamma, beta, eps, a, stats, M, Cc, workspace, workspace_bytes, stream=0):
    _check(lib.hpf_op_bn_relu_forward(dtype, x, gamma, beta, eps, a, stats, M, Cc, workspace, workspace_bytes,
                                      stream or None))


def hpf_op_bn_relu_backward(dtype, x, da, gamma, beta, stats, skip, dx, dgamma, dbeta, M, Cc, workspace,
                            workspace_bytes, stream=0):
    _check(lib.hpf_op_bn_relu_backward(dtype, x, da, gamma, beta, stats, skip or None, dx, dgamma, dbeta, M, Cc,
                                       workspace, workspace_bytes, stream or None))


def hpf_op_bn_relu_forward_noalloc(dtype, x, gamma, beta, eps, a, stats, M, Cc, stream=0):
    _check(lib.hpf_op_bn_relu_forward_noalloc(dtype, x, gamma, beta, eps, a, stats, M, Cc, stream))


def hpf_probe_copy(dst, src, nbytes, stream=0):
    _check(lib.hpf_probe_copy(dst, src, nbytes, stream))


def hpf_probe_mfma_bf16(sink, workgroups, iters, wide=False, stream=0):
    """Returns the flops the launch performs."""
    _check(lib.hpf_probe_mfma_bf16(sink, workgroups, iters, int(wide), stream))
    return float(workgroups) * 4 * iters * 131072


class Ops:
    """Single kernels on torch tensors (tests and kernel benchmarks)."""

    def __init__(self, compute_dtype=HPF_BF16, device="cuda:0"):
        import torch
        self.torch = torch
        self.dt = compute_dtype
        self.tdtype = torch.bfloat16 if compute_dtype == HPF_BF16 else torch.float32
        self.device = torch.device(device)
        self._ws = None

    def workspace(self, cin, cout, R):
        n = hpf_op_workspace_bytes(cin, cout, R)
        if self._ws is None or self._ws.numel() < n + 256:
            self._ws = self.torch.zeros(n + 256, dtype=self.torch.uint8, device=self.device)
        base = (self._ws.data_ptr() + 255) // 256 * 256
        return base, n

    def _s(self):
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def conv_forward(self, x, w, stride=1, add=None, out=None, repack=True):
        b, h, wd, cin = x.shape
        R, _, _, cout = w.shape
        y = out if out is not None else self.torch.empty((b, h // stride, wd // stride, cout), dtype=self.tdtype, device=self.device)
        ws, n = self.workspace(cin, cout, R)
        hpf_op_conv_forward(self.dt, x.data_ptr(), w.data_ptr(), y.data_ptr(), add.data_ptr() if add is not None else 0,
                            b, h, wd, cin, cout, R, stride, ws, n, int(repack), self._s())
        return y

    def conv_dgrad(self, dy, w, in_hw, stride=1, add=None, out=None, repack=True):
        b = dy.shape[0]
        R, _, cin, cout = w.shape
        h, wd = in_hw
        dx = out if out is not None else self.torch.empty((b, h, wd, cin), dtype=self.tdtype, device=self.device)
        ws, n = self.workspace(cin, cout, R)
        hpf_op_conv_dgrad(self.dt, dy.data_ptr(), w.data_ptr(), dx.data_ptr(), add.data_ptr() if add is not None else 0,
                          b, h, wd, cin, cout, R, stride, ws, n, int(repack), self._s())
        return dx

    def conv_wgrad(self, x, dy, R, stride=1, out=None):
        b, h, wd, cin = x.shape
        cout = dy.shape[-1]
        dw = out if out is not None else self.torch.zeros((R, R, cin, cout), dtype=self.torch.float32, device=self.device)
        hpf_op_conv_wgrad(self.dt, x.data_ptr(), dy.data_ptr(), dw.data_ptr(), b, h, wd, cin, cout, R, stride, self._s())
        return dw

    def bn_relu_forward(self, x, gamma, beta, eps=1e-5, out=None):
        Cc = x.shape[-1]
        M = x.numel() // Cc
        a = out if out is not None else self.torch.empty_like(x)
        stats = self.torch.empty(2 * Cc, device=self.device,
                                 dtype=self.torch.float32 if self.dt == HPF_BF16 else self.torch.float64)
        ws, n = self.workspace(Cc, Cc, 1)
        hpf_op_bn_relu_forward(self.dt, x.data_ptr(), gamma.data_ptr(), beta.data_ptr(), eps, a.data_ptr(),
                               stats.data_ptr(), M, Cc, ws, n, self._s())
        return a, stats

    def bn_relu_backward(self, x, da, gamma, beta, stats, skip=None, out=None):
        Cc = x.shape[-1]
        M = x.numel() // Cc
        dx = out if out is not None else self.torch.empty_like(x)
        dg = self.torch.zeros(Cc, dtype=self.torch.float32, device=self.device)
        db = self.torch.zeros(Cc, dtype=self.torch.float32, device=self.device)
        ws, n = self.workspace(Cc, Cc, 1)
        hpf_op_bn_relu_backward(self.dt, x.data_ptr(), da.data_ptr(), gamma.data_ptr(), beta.data_ptr(), stats.data_ptr(),
                                skip.data_ptr() if skip is not None else 0, dx.data_ptr(), dg.data_ptr(), db.data_ptr(),
                                M, Cc, ws, n, self._s())
        return dx, dg, db


class Partition:
    """One partition on the current torch device.  torch supplies device memory and streams."""

    def __init__(self, spec, params, compute_dtype=HPF_BF16, device="cuda:0"):
        import numpy as np
        import torch
        self.torch = torch
        self.spec = spec
        self.compute_dtype = compute_dtype
        self.tdtype = torch.bfloat16 if compute_dtype == HPF_BF16 else torch.float32
        self.device = torch.device(device)
        self.desc, self._keep = make_desc(spec, compute_dtype)
        self.sizes = hpf_partition_sizes(self.desc)
        params = np.ascontiguousarray(params, dtype=np.float32)
        if params.size != self.sizes.n_params:
            raise ValueError(f"expected {self.sizes.n_params} parameters, got {params.size}")
        self.n_params = int(self.sizes.n_params)
        self.arena = torch.empty(int(self.sizes.arena_bytes) + 256, dtype=torch.uint8, device=self.device)
        base = (self.arena.data_ptr() + 255) // 256 * 256
        with torch.cuda.device(self.device):
            self.handle = hpf_partition_create(self.desc, base, int(self.sizes.arena_bytes), params)
        oh, ow, oc = spec.out_shape()
        self.in_shape = (spec.microbatch, spec.in_h, spec.in_w, spec.in_c)
        self.out_shape = (spec.microbatch, oh, ow, oc)
        self.in_dtype = torch.float32 if spec.has_stem else self.tdtype
        self.skip_in_shape = (spec.microbatch,) + tuple(spec.skip_in_shape()) if getattr(spec, "has_skip_in", False) else None
        self.skip_out_shape = (spec.microbatch,) + tuple(spec.skip_out_shape()) if getattr(spec, "has_skip_out", False) else None
        self.loss = torch.zeros(1, dtype=torch.float32, device=self.device)

    def close(self):
        if getattr(self, "handle", None):
            hpf_partition_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _stream(stream):
        if stream is None:
            return 0
        return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)

    def _stream_or_current(self, stream):
        return self._stream(stream if stream is not None else self.torch.cuda.current_stream(self.device))

    def forward_microbatch(self, mb, act_in, labels=None, act_out=None, stream=None):
        assert tuple(act_in.shape) == self.in_shape and act_in.dtype == self.in_dtype and act_in.is_contiguous()
        if self.spec.has_head:
            assert labels is not None and labels.dtype == self.torch.int32 and labels.numel() == self.spec.microbatch
        else:
            if act_out is None:
                act_out = self.torch.empty(self.out_shape, dtype=self.tdtype, device=self.device)
            assert tuple(act_out.shape) == self.out_shape and act_out.dtype == self.tdtype and act_out.is_contiguous()
        hpf_forward_microbatch(self.handle, mb, act_in.data_ptr(),
                               labels.data_ptr() if labels is not None else 0,
                               act_out.data_ptr() if act_out is not None else 0,
                               self.loss.data_ptr() if self.spec.has_head else 0,
                               self._stream_or_current(stream))
        return act_out

    def backward_microbatch(self, mb, err_in=None, err_out=None, stream=None):
        if not self.spec.has_head:
            assert tuple(err_in.shape) == self.out_shape and err_in.dtype == self.tdtype and err_in.is_contiguous()
        if not self.spec.has_stem:
            if err_out is None:
                err_out = self.torch.empty(self.in_shape, dtype=self.tdtype, device=self.device)
            assert tuple(err_out.shape) == self.in_shape and err_out.dtype == self.tdtype and err_out.is_contiguous()
        hpf_backward_microbatch(self.handle, mb, err_in.data_ptr() if err_in is not None else 0,
                                err_out.data_ptr() if err_out is not None else 0, self._stream_or_current(stream))
        return err_out

    def _skip_ok(self, t, shape):
        return t is not None and tuple(t.shape) == shape and t.dtype == self.tdtype and t.is_contiguous()

    def forward_microbatch_cut(self, mb, act_in, skip_in=None, labels=None, act_out=None, skip_out=None, stream=None):
        """Forward of a partition cut at layer granularity: returns (act_out, skip_out)."""
        assert tuple(act_in.shape) == self.in_shape and act_in.dtype == self.in_dtype and act_in.is_contiguous()
        if not self.spec.has_head and act_out is None:
            act_out = self.torch.empty(self.out_shape, dtype=self.tdtype, device=self.device)
        if self.skip_in_shape:
            assert self._skip_ok(skip_in, self.skip_in_shape)
        if self.skip_out_shape:
            if skip_out is None:
                skip_out = self.torch.empty(self.skip_out_shape, dtype=self.tdtype, device=self.device)
            assert self._skip_ok(skip_out, self.skip_out_shape)
        hpf_forward_microbatch_cut(self.handle, mb, act_in.data_ptr(), skip_in.data_ptr() if skip_in is not None else 0,
                                   labels.data_ptr() if labels is not None else 0,
                                   act_out.data_ptr() if act_out is not None else 0,
                                   skip_out.data_ptr() if skip_out is not None else 0,
                                   self.loss.data_ptr() if self.spec.has_head else 0, self._stream_or_current(stream))
        return act_out, skip_out

    def backward_microbatch_cut(self, mb, err_in=None, skip_err_in=None, err_out=None, skip_err_out=None, stream=None):
        """Backward of a partition cut at layer granularity: returns (err_out, skip_err_out)."""
        if not self.spec.has_stem and err_out is None:
            err_out = self.torch.empty(self.in_shape, dtype=self.tdtype, device=self.device)
        if self.skip_out_shape:
            assert self._skip_ok(skip_err_in, self.skip_out_shape)
        if self.skip_in_shape:
            if skip_err_out is None:
                skip_err_out = self.torch.empty(self.skip_in_shape, dtype=self.tdtype, device=self.device)
            assert self._skip_ok(skip_err_out, self.skip_in_shape)
        hpf_backward_microbatch_cut(self.handle, mb, err_in.data_ptr() if err_in is not None else 0,
                                    skip_err_in.data_ptr() if skip_err_in is not None else 0,
                                    err_out.data_ptr() if err_out is not None else 0,
                                    skip_err_out.data_ptr() if skip_err_out is not None else 0,
                                    self._stream_or_current(stream))
        return err_out, skip_err_out

    def forward_microbatches(self, mb_first, act_in, labels=None, act_out=None, stream=None):
        """Group call: lists of tensors for micro-batches mb_first, mb_first+1, ..."""
        n = len(act_in)
        for t in act_in:
            assert tuple(t.shape) == self.in_shape and t.dtype == self.in_dtype and t.is_contiguous()
        if self.spec.has_head:
            assert labels is not None and len(labels) == n
        else:
            if act_out is None:
                act_out = [self.torch.empty(self.out_shape, dtype=self.tdtype, device=self.device) for _ in range(n)]
            for t in act_out:
                assert tuple(t.shape) == self.out_shape and t.dtype == self.tdtype and t.is_contiguous()
        hpf_forward_microbatches(self.handle, mb_first, [t.data_ptr() for t in act_in],
                                 [t.data_ptr() for t in labels] if labels is not None else None,
                                 [t.data_ptr() for t in act_out] if act_out is not None else None,
                                 self.loss.data_ptr() if self.spec.has_head else 0, self._stream_or_current(stream))
        return act_out

    def backward_microbatches(self, mb_first, count, err_in=None, err_out=None, stream=None):
        if not self.spec.has_head:
            assert len(err_in) == count
            for t in err_in:
                assert tuple(t.shape) == self.out_shape and t.dtype == self.tdtype and t.is_contiguous()
        if not self.spec.has_stem:
            if err_out is None:
                err_out = [self.torch.empty(self.in_shape, dtype=self.tdtype, device=self.device) for _ in range(count)]
            for t in err_out:
                assert tuple(t.shape) == self.in_shape and t.dtype == self.tdtype and t.is_contiguous()
        hpf_backward_microbatches(self.handle, mb_first, count,
                                  [t.data_ptr() for t in err_in] if err_in is not None else None,
                                  [t.data_ptr() for t in err_out] if err_out is not None else None,
                                  self._stream_or_current(stream))
        return err_out

    def grad_accum_read(self, out=None, stream=None):
        """Returns the accumulated gradient: into a device tensor `out` (async) or as a numpy array."""
        if out is not None:
            assert out.dtype == self.torch.float32 and out.numel() == self.n_params and out.is_contiguous()
            hpf_grad_accum_read(self.handle, out.data_ptr(), self.n_params, True, self._stream_or_current(stream))
            return out
        import numpy as np
        g = np.empty(self.n_params, np.float32)
        hpf_grad_accum_read(self.handle, g.ctypes.data, self.n_params, False, self._stream_or_current(stream))
        return g

    def grad_accum_zero(self, stream=None):
        hpf_grad_accum_zero(self.handle, self._stream_or_current(stream))

    def sgd_step(self, lr, momentum, stream=None):
        hpf_sgd_step(self.handle, lr, momentum, self._stream_or_current(stream))

    def set_graphs(self, enable):
        hpf_partition_set_graphs(self.handle, enable)

    def set_fusion(self, level):
        hpf_partition_set_fusion(self.handle, level)

    def set_profiling(self, enable):
        hpf_partition_set_profiling(self.handle, enable)

    def set_bn_momentum(self, momentum):
        hpf_partition_set_bn_momentum(self.handle, momentum)

    def bn_running_read(self):
        import numpy as np
        r = np.empty(int(self.sizes.n_bn_running), np.float32)
        hpf_bn_running_read(self.handle, r.ctypes.data, r.size)
        return r

    def bn_running_write(self, r):
        import numpy as np
        r = np.ascontiguousarray(r, np.float32)
        hpf_bn_running_write(self.handle, r.ctypes.data, r.size)

    def forward_inference(self, act_in, skip_in=None, stream=None, out=None):
        """Inference forward: logits [b, classes] fp32 with a head, else act_out (or (act_out, skip_out))."""
        torch = self.torch
        assert tuple(act_in.shape) == self.in_shape and act_in.dtype == self.in_dtype and act_in.is_contiguous()
        if out is not None:
            assert out.is_contiguous() and out.numel() == (self.spec.microbatch * self.spec.num_classes if self.spec.has_head
                                                           else int(self.sizes.act_out_elems))
        elif self.spec.has_head:
            out = torch.empty((self.spec.microbatch, self.spec.num_classes), dtype=torch.float32, device=self.device)
        else:
            out = torch.empty(self.out_shape, dtype=self.tdtype, device=self.device)
        skip_out = torch.empty(self.skip_out_shape, dtype=self.tdtype, device=self.device) if self.skip_out_shape else None
        if self.skip_in_shape:
            assert self._skip_ok(skip_in, self.skip_in_shape)
        hpf_forward_inference(self.handle, act_in.data_ptr(), skip_in.data_ptr() if skip_in is not None else 0, out.data_ptr(),
                              skip_out.data_ptr() if skip_out is not None else 0, self._stream_or_current(stream))
        return (out, skip_out) if skip_out is not None else out

    def forward_inference_group(self, act_in, skip_in=None, stream=None, out=None):
        """Inference forward of several micro-batches in one call: list of outputs (or of (act_out, skip_out)).
        out: optional list of output tensors to write into (the same tensors every call let the library replay
        one HIP graph)."""
        torch = self.torch
        n = len(act_in)
        for t in act_in:
            assert tuple(t.shape) == self.in_shape and t.dtype == self.in_dtype and t.is_contiguous()
        shape = (self.spec.microbatch, self.spec.num_classes) if self.spec.has_head else self.out_shape
        dt = torch.float32 if self.spec.has_head else self.tdtype
        outs = out if out is not None else [torch.empty(shape, dtype=dt, device=self.device) for _ in range(n)]
        assert len(outs) == n and all(tuple(t.shape) == shape and t.dtype == dt and t.is_contiguous() for t in outs)
        skos = [torch.empty(self.skip_out_shape, dtype=self.tdtype, device=self.device) for _ in range(n)] if self.skip_out_shape else None
        if self.skip_in_shape:
            assert skip_in is not None and all(self._skip_ok(t, self.skip_in_shape) for t in skip_in)
        hpf_forward_inference_group(self.handle, [t.data_ptr() for t in act_in],
                                    [t.data_ptr() for t in skip_in] if skip_in is not None else None,
                                    [t.data_ptr() for t in outs], [t.data_ptr() for t in skos] if skos else None,
                                    self._stream_or_current(stream))
        return list(zip(outs, skos)) if skos else outs

    def profile_read(self):
        """[{name, launches, total_ms, bytes_per_launch, flops_per_launch}] since profiling was enabled."""
        return hpf_partition_profile_read(self.handle)

    def stash_read(self, mb, unit, tensor):
        """One stashed tensor of micro-batch mb as a flat float32 array (statistics: float64), or the name of the
        caller buffer that holds it ("act_in", "err_out", ...)."""
        import numpy as np
        torch = self.torch
        where, need = hpf_stash_read(self.handle, mb, unit, tensor, None, 0)
        if where != 0:
            return STASH_WHERE[where]
        raw = np.empty(need, np.uint8)
        hpf_stash_read(self.handle, mb, unit, tensor, raw.ctypes.data, need)
        if HPF_T_STATS0 <= tensor <= HPF_T_STATS2:
            return raw.view(np.float32 if self.compute_dtype == HPF_BF16 else np.float64).astype(np.float64)
        if self.compute_dtype == HPF_BF16:
            return torch.from_numpy(raw.view(np.int16)).view(torch.bfloat16).float().numpy()
        return raw.view(np.float32).copy()

    def check(self):
        """Waits for the device; raises HpfError(HPF_EDEVICE) if the handle's results are marked invalid."""
        hpf_partition_check(self.handle)

    def params_read(self):
        import numpy as np
        p = np.empty(self.n_params, np.float32)
        hpf_params_read(self.handle, p.ctypes.data, self.n_params)
        return p
