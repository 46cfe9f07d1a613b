"""Thin ctypes binding of libswconv.so: the same entry points as include/swconv.h, argument
marshalling only.  Every step of the forward pass runs in the library's HIP kernels; there is no
fallback: a missing library raises."""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

SWCONV_OK, SWCONV_EINVAL, SWCONV_EUNSUPPORTED, SWCONV_ENOMEM, SWCONV_EHIP, SWCONV_ESTATE = range(6)

EXPORTS = [
    "swconv_status_string", "swconv_plan_create", "swconv_plan_destroy", "swconv_set_weights",
    "swconv_forward", "swconv_set_weights_dense", "swconv_forward_dense", "swconv_profile_forward",
    "swconv_debug_copy_V", "swconv_debug_copy_M", "swconv_debug_export_weights", "swconv_plan_sizes",
    "swconv_plan_weight_stats", "swconv_debug_check_schedule",
    "swconv_backward", "swconv_debug_copy_dZ", "swconv_debug_copy_dV", "swconv_profile_backward",
    "swconv_prune_step", "swconv_set_weights_device", "swconv_plan_set_image_strides",
    "swconv_update_values", "swconv_forward_noalloc",
]

_lib = None
_i32p = ctypes.POINTER(ctypes.c_int32)
_f32p = ctypes.POINTER(ctypes.c_float)
_vp = ctypes.c_void_p


class SwconvError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s" % (where, swconv_status_string(status)))


def lib():
    """Load libswconv.so (building it only if no built library is present)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build_library()
        L = ctypes.CDLL(_build.LIB)
        L.swconv_status_string.restype = ctypes.c_char_p
        L.swconv_status_string.argtypes = [ctypes.c_int]
        L.swconv_plan_create.argtypes = [ctypes.POINTER(_vp)] + [ctypes.c_int] * 8
        L.swconv_plan_destroy.argtypes = [_vp]
        L.swconv_plan_destroy.restype = None
        L.swconv_set_weights.argtypes = [_vp, _i32p, _i32p, _f32p]
        L.swconv_forward.argtypes = [_vp, _vp, _vp, _vp]
        L.swconv_forward_noalloc.argtypes = [_vp, _vp, _vp, _vp]
        L.swconv_set_weights_dense.argtypes = [_vp, _f32p]
        L.swconv_forward_dense.argtypes = [_vp, _vp, _vp, _vp]
        L.swconv_profile_forward.argtypes = [_vp, _vp, _vp, _vp, ctypes.c_int, _f32p]
        L.swconv_debug_copy_V.argtypes = [_vp, _f32p]
        L.swconv_debug_copy_M.argtypes = [_vp, _f32p]
        L.swconv_debug_export_weights.argtypes = [_vp, _i32p, _i32p, _f32p]
        L.swconv_plan_sizes.argtypes = [_vp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int64),
                                        ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.swconv_plan_weight_stats.argtypes = [_vp, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64),
                                               ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int64)]
        L.swconv_debug_check_schedule.argtypes = [_vp]
        L.swconv_plan_set_image_strides.argtypes = [_vp, ctypes.c_int64, ctypes.c_int64]
        L.swconv_update_values.argtypes = [_vp, _vp, _vp]
        L.swconv_backward.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp]
        L.swconv_profile_backward.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_int, _f32p]
        L.swconv_prune_step.argtypes = [ctypes.c_int64, _vp, _vp, _vp, _vp] + [ctypes.c_float] * 4 + [_vp] * 5
        L.swconv_set_weights_device.argtypes = [_vp] * 5
        L.swconv_debug_copy_dZ.argtypes = [_vp, _f32p]
        L.swconv_debug_copy_dV.argtypes = [_vp, _f32p]
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None and a.size else None


def _check(status, where):
    if status != SWCONV_OK:
        raise SwconvError(status, where)


def swconv_status_string(status):
    return lib().swconv_status_string(int(status)).decode()


def swconv_plan_create(N, C, H, W, K, m, r, pad):
    """-> opaque plan handle (int).  Raises SwconvError with the library's status."""
    h = _vp()
    _check(lib().swconv_plan_create(ctypes.byref(h), N, C, H, W, K, m, r, pad), "swconv_plan_create")
    return h


def swconv_plan_destroy(plan):
    lib().swconv_plan_destroy(plan)


def swconv_set_weights(plan, rowptr, colidx, vals):
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    _check(lib().swconv_set_weights(plan, rowptr.ctypes.data_as(_i32p), _p(colidx, ctypes.c_int32),
                                    _p(vals, ctypes.c_float)), "swconv_set_weights")


def swconv_set_weights_status(plan, rowptr, colidx, vals):
    """Same call, returning the raw status instead of raising (for error-path tests)."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    return lib().swconv_set_weights(plan, rowptr.ctypes.data_as(_i32p), _p(colidx, ctypes.c_int32),
                                    _p(vals, ctypes.c_float))


def swconv_forward(plan, stream, in_dev_ptr, out_dev_ptr):
    """stream: hipStream_t as int (0 = default); in/out: device addresses as int."""
    _check(lib().swconv_forward(plan, _vp(stream), _vp(in_dev_ptr), _vp(out_dev_ptr)), "swconv_forward")


def swconv_forward_noalloc(plan, stream, in_dev_ptr, out_dev_ptr):
    """swconv_forward with the intermediates in the library's static device scratch (no allocation)."""
    _check(lib().swconv_forward_noalloc(plan, _vp(stream), _vp(in_dev_ptr), _vp(out_dev_ptr)), "swconv_forward_noalloc")


def swconv_backward(plan, stream, in_dev_ptr, dout_dev_ptr, din_dev_ptr, dvals_dev_ptr):
    """Device addresses as int; din_dev_ptr / dvals_dev_ptr may be 0 (not wanted)."""
    _check(lib().swconv_backward(plan, _vp(stream), _vp(in_dev_ptr), _vp(dout_dev_ptr), _vp(din_dev_ptr or None),
                                 _vp(dvals_dev_ptr or None)), "swconv_backward")


def swconv_prune_step(rows, rowptr_dev, colidx_dev, vals_dev, grad_dev, eta, lam, eps, beta, stream, updated_dev,
                      rowptr_out_dev, colidx_out_dev, vals_out_dev):
    """Device addresses as int."""
    _check(lib().swconv_prune_step(int(rows), _vp(rowptr_dev), _vp(colidx_dev), _vp(vals_dev), _vp(grad_dev),
                                   float(eta), float(lam), float(eps), float(beta), _vp(stream), _vp(updated_dev),
                                   _vp(rowptr_out_dev), _vp(colidx_out_dev), _vp(vals_out_dev)), "swconv_prune_step")


def swconv_set_weights_device(plan, stream, rowptr_dev, colidx_dev, vals_dev):
    _check(lib().swconv_set_weights_device(plan, _vp(stream), _vp(rowptr_dev), _vp(colidx_dev), _vp(vals_dev)),
           "swconv_set_weights_device")


BACKWARD_STAGES = ("output_grad_transform_kernel", "input_transform_kernel", "spmm_kernel<sampled>",
                   "weight_grad_reduce_kernel", "spmm_kernel<transposed>", "input_grad_patch_kernel",
                   "input_grad_gather_kernel")


def swconv_profile_backward(plan, stream, in_dev_ptr, dout_dev_ptr, din_dev_ptr, dvals_dev_ptr, iters):
    """-> numpy float32[7]: mean milliseconds of each backward kernel, in launch order (BACKWARD_STAGES)."""
    ms = np.zeros(7, dtype=np.float32)
    _check(lib().swconv_profile_backward(plan, _vp(stream), _vp(in_dev_ptr), _vp(dout_dev_ptr),
                                         _vp(din_dev_ptr or None), _vp(dvals_dev_ptr or None), int(iters),
                                         ms.ctypes.data_as(_f32p)), "swconv_profile_backward")
    return ms


def swconv_debug_copy_dZ(plan, K):
    P, T, _, _ = swconv_plan_sizes(plan)
    dZ = np.empty((P, K, T), dtype=np.float32)
    _check(lib().swconv_debug_copy_dZ(plan, dZ.ctypes.data_as(_f32p)), "swconv_debug_copy_dZ")
    return dZ


def swconv_debug_copy_dV(plan, C):
    P, T, _, _ = swconv_plan_sizes(plan)
    dV = np.empty((P, C, T), dtype=np.float32)
    _check(lib().swconv_debug_copy_dV(plan, dV.ctypes.data_as(_f32p)), "swconv_debug_copy_dV")
    return dV


def swconv_set_weights_dense(plan, wf):
    wf = np.ascontiguousarray(wf, dtype=np.float32)
    _check(lib().swconv_set_weights_dense(plan, wf.ctypes.data_as(_f32p)), "swconv_set_weights_dense")


def swconv_forward_dense(plan, stream, in_dev_ptr, out_dev_ptr):
    _check(lib().swconv_forward_dense(plan, _vp(stream), _vp(in_dev_ptr), _vp(out_dev_ptr)), "swconv_forward_dense")


def swconv_profile_forward(plan, stream, in_dev_ptr, out_dev_ptr, iters):
    """-> numpy float32[3]: mean milliseconds of the input transform, sparse product, output transform."""
    ms = np.zeros(3, dtype=np.float32)
    _check(lib().swconv_profile_forward(plan, _vp(stream), _vp(in_dev_ptr), _vp(out_dev_ptr), int(iters),
                                        ms.ctypes.data_as(_f32p)), "swconv_profile_forward")
    return ms


def swconv_update_values(plan, stream, vals_dev_ptr):
    _check(lib().swconv_update_values(plan, _vp(stream), _vp(vals_dev_ptr)), "swconv_update_values")


def swconv_plan_set_image_strides(plan, in_stride, out_stride):
    _check(lib().swconv_plan_set_image_strides(plan, int(in_stride), int(out_stride)), "swconv_plan_set_image_strides")


def swconv_plan_sizes(plan):
    P, T, Ho, Wo = ctypes.c_int(), ctypes.c_int64(), ctypes.c_int(), ctypes.c_int()
    _check(lib().swconv_plan_sizes(plan, ctypes.byref(P), ctypes.byref(T), ctypes.byref(Ho), ctypes.byref(Wo)),
           "swconv_plan_sizes")
    return P.value, T.value, Ho.value, Wo.value


def swconv_plan_weight_stats(plan):
    a, b, c, d = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int(), ctypes.c_int64()
    _check(lib().swconv_plan_weight_stats(plan, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(d)),
           "swconv_plan_weight_stats")
    return dict(nnz=a.value, padded_nnz=b.value, work_items=c.value, max_item=d.value)


def swconv_debug_check_schedule(plan):
    """Raises unless the sparse product's static schedule covers every unit exactly once."""
    _check(lib().swconv_debug_check_schedule(plan), "swconv_debug_check_schedule")


def swconv_debug_copy_V(plan, C):
    P, T, _, _ = swconv_plan_sizes(plan)
    V = np.empty((P, C, T), dtype=np.float32)
    _check(lib().swconv_debug_copy_V(plan, V.ctypes.data_as(_f32p)), "swconv_debug_copy_V")
    return V


def swconv_debug_copy_M(plan, K):
    P, T, _, _ = swconv_plan_sizes(plan)
    M = np.empty((P, K, T), dtype=np.float32)
    _check(lib().swconv_debug_copy_M(plan, M.ctypes.data_as(_f32p)), "swconv_debug_copy_M")
    return M


def swconv_debug_export_weights(plan, K, nnz):
    P, _, _, _ = swconv_plan_sizes(plan)
    rowptr = np.empty(P * K + 1, dtype=np.int32)
    colidx = np.empty(nnz, dtype=np.int32)
    vals = np.empty(nnz, dtype=np.float32)
    _check(lib().swconv_debug_export_weights(plan, rowptr.ctypes.data_as(_i32p), _p(colidx, ctypes.c_int32),
                                             _p(vals, ctypes.c_float)), "swconv_debug_export_weights")
    return rowptr, colidx, vals
