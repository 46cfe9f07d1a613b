"""ctypes front-end of the CPU oracle (``swconv_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU package never imports this module and this
module never imports the GPU package.

The functions mirror the C entry points; array shapes follow the paper's Eq. 4
(Section 3) with positions ``p = i*t + j`` and tiles ``tau = (n*th + ty)*tw + tx``:

* ``forward_f64`` / ``forward_f32`` -> ``(out, V, M)`` with ``V[P][C][T]``,
  ``M[P][K][T]`` and ``out[N][K][Ho][Wo]``.
* ``direct_conv_f64`` -> Eq. 1 (cross-correlation, zero padding).
* ``wf_from_spatial_f64`` -> ``W_F = G w G^T`` (Eq. 3) as ``[P][K][C]``.
* ``winograd_matrices`` -> ``(AT, BT, G)``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "swconv_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ -O2 -fopenmp (no intrinsics, no BLAS)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["g++", "-O2", "-ffp-contract=off", "-std=c++17", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f64p = ctypes.POINTER(ctypes.c_double)
        f32p = ctypes.POINTER(ctypes.c_float)
        ints8 = [ctypes.c_int] * 8
        lib.oracle_forward_f64.argtypes = ints8 + [f64p, i32p, i32p, f64p, f64p, f64p, f64p]
        lib.oracle_forward_f32.argtypes = ints8 + [f32p, i32p, i32p, f32p, f32p, f32p, f32p]
        lib.oracle_backward_f64.argtypes = ints8 + [f64p, i32p, i32p, f64p, f64p, f64p, f64p, f64p, f64p]
        lib.oracle_backward_f32.argtypes = ints8 + [f32p, i32p, i32p, f32p, f32p, f32p, f32p, f32p, f32p]
        for fn, fp, ct in ((lib.oracle_prune_step_f32, f32p, ctypes.c_float), (lib.oracle_prune_step_f64, f64p, ctypes.c_double)):
            fn.argtypes = [ctypes.c_int64, i32p, i32p, fp, fp, ct, ct, ct, ct, fp, i32p, i32p, fp]
            fn.restype = ctypes.c_int64
        lib.oracle_direct_conv_f64.argtypes = [ctypes.c_int] * 7 + [f64p, f64p, f64p]
        lib.oracle_wf_from_spatial_f64.argtypes = [ctypes.c_int] * 4 + [f64p, f64p]
        lib.oracle_winograd_matrices.argtypes = [ctypes.c_int] * 2 + [f64p, f64p, f64p]
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        lib.oracle_set_num_threads.restype = None
        _lib = lib
    return _lib


def _ptr(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def out_shape(N, C, H, W, K, m, r, pad):
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    th, tw = -(-Ho // m), -(-Wo // m)
    return Ho, Wo, th, tw, N * th * tw


def _forward(fn, dt, ct, inp, rowptr, colidx, vals, K, m, r, pad, want_VM):
    inp = np.ascontiguousarray(inp, dtype=dt)
    N, C, H, W = inp.shape
    Ho, Wo, th, tw, T = out_shape(N, C, H, W, K, m, r, pad)
    t = m + r - 1
    P = t * t
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=dt)
    assert rowptr.shape == (P * K + 1,)
    assert colidx.shape == vals.shape == (int(rowptr[-1]),)
    out = np.zeros((N, K, Ho, Wo), dtype=dt)
    V = np.empty((P, C, T), dtype=dt) if want_VM else None
    M = np.empty((P, K, T), dtype=dt) if want_VM else None
    rc = fn(N, C, H, W, K, m, r, pad, _ptr(inp, ct), _ptr(rowptr, ctypes.c_int32),
            _ptr(colidx, ctypes.c_int32), _ptr(vals, ct), _ptr(V, ct), _ptr(M, ct), _ptr(out, ct))
    if rc != 0:
        raise ValueError("oracle forward failed with status %d" % rc)
    return out, V, M


def forward_f64(inp, rowptr, colidx, vals, K, m, r=3, pad=1, want_VM=True):
    """Eq. 4 in double precision (inputs are promoted exactly)."""
    return _forward(_load().oracle_forward_f64, np.float64, ctypes.c_double, inp, rowptr, colidx,
                    vals, K, m, r, pad, want_VM)


def forward_f32(inp, rowptr, colidx, vals, K, m, r=3, pad=1, want_VM=False):
    """The same loops in float: the timed CPU baseline."""
    return _forward(_load().oracle_forward_f32, np.float32, ctypes.c_float, inp, rowptr, colidx,
                    vals, K, m, r, pad, want_VM)


def _backward(fn, dt, ct, inp, rowptr, colidx, vals, dout, K, m, r, pad, want_ZV):
    inp = np.ascontiguousarray(inp, dtype=dt)
    N, C, H, W = inp.shape
    Ho, Wo, th, tw, T = out_shape(N, C, H, W, K, m, r, pad)
    t = m + r - 1
    P = t * t
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=dt)
    dout = np.ascontiguousarray(dout, dtype=dt)
    assert rowptr.shape == (P * K + 1,) and dout.shape == (N, K, Ho, Wo)
    assert colidx.shape == vals.shape == (int(rowptr[-1]),)
    din = np.empty((N, C, H, W), dtype=dt)
    dvals = np.empty(vals.shape, dtype=dt)
    dZ = np.empty((P, K, T), dtype=dt) if want_ZV else None
    dV = np.empty((P, C, T), dtype=dt) if want_ZV else None
    rc = fn(N, C, H, W, K, m, r, pad, _ptr(inp, ct), _ptr(rowptr, ctypes.c_int32), _ptr(colidx, ctypes.c_int32),
            _ptr(vals, ct), _ptr(dout, ct), _ptr(dZ, ct), _ptr(dV, ct), _ptr(dvals, ct), _ptr(din, ct))
    if rc != 0:
        raise ValueError("oracle backward failed with status %d" % rc)
    return din, dvals, dZ, dV


def backward_f64(inp, rowptr, colidx, vals, dout, K, m, r=3, pad=1, want_ZV=True):
    """Eq. 5 and Eq. 6 in double precision: (dL/dI, dL/dW_F at the stored entries, dL/dZ, dL/dI_F)."""
    return _backward(_load().oracle_backward_f64, np.float64, ctypes.c_double, inp, rowptr, colidx, vals, dout, K, m,
                     r, pad, want_ZV)


def backward_f32(inp, rowptr, colidx, vals, dout, K, m, r=3, pad=1, want_ZV=False):
    """The same loops in float: the timed CPU baseline of the backward pass."""
    return _backward(_load().oracle_backward_f32, np.float32, ctypes.c_float, inp, rowptr, colidx, vals, dout, K, m,
                     r, pad, want_ZV)


def prune_step(rowptr, colidx, vals, grad, eta, lam, eps=1e-4, beta=0.1, dtype=np.float32):
    """Eq. 9 + Eq. 8 on the stored entries: -> (updated values in the old pattern, (rowptr, colidx, vals) of the
    kept entries).  dtype float32 takes every rounding and the keep/drop decision in float, as the GPU kernel does."""
    dt = np.dtype(dtype)
    ct = ctypes.c_float if dt == np.float32 else ctypes.c_double
    fn = _load().oracle_prune_step_f32 if dt == np.float32 else _load().oracle_prune_step_f64
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=dt)
    grad = np.ascontiguousarray(grad, dtype=dt)
    assert vals.shape == grad.shape == colidx.shape == (int(rowptr[-1]),)
    updated = np.empty_like(vals)
    rp = np.empty_like(rowptr)
    ci = np.empty_like(colidx)
    va = np.empty_like(vals)
    kept = fn(len(rowptr) - 1, _ptr(rowptr, ctypes.c_int32), _ptr(colidx, ctypes.c_int32), _ptr(vals, ct),
              _ptr(grad, ct), ct(eta), ct(lam), ct(eps), ct(beta), _ptr(updated, ct), _ptr(rp, ctypes.c_int32),
              _ptr(ci, ctypes.c_int32), _ptr(va, ct))
    return updated, (rp, ci[:kept].copy(), va[:kept].copy())


def direct_conv_f64(inp, w, pad):
    """Eq. 1, cross-correlation with zero padding; w is [K][C][r][r]."""
    inp = np.ascontiguousarray(inp, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    N, C, H, W = inp.shape
    K, C2, r, r2 = w.shape
    assert C2 == C and r2 == r
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    out = np.zeros((N, K, Ho, Wo), dtype=np.float64)
    rc = _load().oracle_direct_conv_f64(N, C, H, W, K, r, pad, _ptr(inp, ctypes.c_double),
                                        _ptr(w, ctypes.c_double), _ptr(out, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle direct conv failed with status %d" % rc)
    return out


def wf_from_spatial_f64(w, m):
    """W_F[p][k][c] = (G w[k][c] G^T)[i][j] with p = i*t + j (Eq. 3)."""
    w = np.ascontiguousarray(w, dtype=np.float64)
    K, C, r, _ = w.shape
    t = m + r - 1
    wf = np.empty((t * t, K, C), dtype=np.float64)
    rc = _load().oracle_wf_from_spatial_f64(K, C, m, r, _ptr(w, ctypes.c_double),
                                            _ptr(wf, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle weight transform failed with status %d" % rc)
    return wf


def winograd_matrices(m, r=3):
    t = m + r - 1
    AT = np.empty((m, t))
    BT = np.empty((t, t))
    G = np.empty((t, r))
    rc = _load().oracle_winograd_matrices(m, r, _ptr(AT, ctypes.c_double),
                                          _ptr(BT, ctypes.c_double), _ptr(G, ctypes.c_double))
    if rc != 0:
        raise ValueError("unsupported F(%d,%d)" % (m, r))
    return AT, BT, G


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))
