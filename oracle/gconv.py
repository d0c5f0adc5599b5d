"""CPU oracle for group-convolution training (more than one channel per group).

TEST INFRASTRUCTURE ONLY: the slow fp64 checker for the GPU library's group-convolution entry
points.  Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module;
the GPU package never does.

The arithmetic lives in ``gconv_oracle.c`` (plain loop nests writing out the definition of a group
convolution; paper Section V-B: depthwise convolution is the special case with as many groups as
channels).  This module compiles that file with gcc and marshals numpy arrays into it.
``dense_group_*`` below is a second, separately written route to the same results: the standard
im2col + dense product of Section II with the weight matrix masked group-wise (the 0/1 mask of
Section III-A, Eq. 2, with one block per pair of channels of the same group), used to pin the loop
nests on tiny inputs.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

from .dense_identity import col2im, im2col

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gconv_oracle.c")
_LIB = os.path.join(_HERE, "libgconv_oracle.so")
_lock = threading.Lock()
_lib = None

NCHW = 0
NHWC = 1


class _Desc(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in
                ("N", "C", "H", "W", "K", "stride", "pad", "groups", "O", "layout")]


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            dp = ctypes.POINTER(ctypes.c_double)
            for name in ("oracle_gconv_fwd", "oracle_gconv_bwd_data", "oracle_gconv_bwd_filter"):
                fn = getattr(lib, name)
                fn.argtypes = [ctypes.POINTER(_Desc), dp, dp, dp, ctypes.c_int]
                fn.restype = ctypes.c_int
            lib.oracle_gconv_out_dims.argtypes = [ctypes.POINTER(_Desc), ctypes.POINTER(ctypes.c_int32),
                                                  ctypes.POINTER(ctypes.c_int32)]
            lib.oracle_gconv_out_dims.restype = ctypes.c_int
            _lib = lib
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _shapes(x_shape, K, stride, pad, groups, O, layout):
    if layout == NCHW:
        N, C, H, W = x_shape
    else:
        N, H, W, C = x_shape
    d = _Desc(int(N), int(C), int(H), int(W), int(K), int(stride), int(pad), int(groups), int(O), int(layout))
    ho, wo = ctypes.c_int32(0), ctypes.c_int32(0)
    if _load().oracle_gconv_out_dims(ctypes.byref(d), ctypes.byref(ho), ctypes.byref(wo)):
        raise ValueError("invalid group-convolution shape")
    Cg = C // groups
    yshape = (N, O, ho.value, wo.value) if layout == NCHW else (N, ho.value, wo.value, O)
    wshape = (O, Cg, K, K) if layout == NCHW else (K, K, Cg, O)
    return d, yshape, wshape


def fwd(x, w, *, K, stride=1, pad=0, groups, O, layout=NCHW, nthreads=1):
    x = _f64(x); w = _f64(w)
    d, yshape, wshape = _shapes(x.shape, K, stride, pad, groups, O, layout)
    assert w.shape == wshape, (w.shape, wshape)
    y = np.empty(yshape, dtype=np.float64)
    assert _load().oracle_gconv_fwd(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(y), int(nthreads)) == 0
    return y


def bwd_data(dy, w, *, x_shape, K, stride=1, pad=0, groups, O, layout=NCHW, nthreads=1):
    dy = _f64(dy); w = _f64(w)
    d, yshape, wshape = _shapes(tuple(x_shape), K, stride, pad, groups, O, layout)
    assert dy.shape == yshape, (dy.shape, yshape)
    assert w.shape == wshape, (w.shape, wshape)
    dx = np.empty(tuple(x_shape), dtype=np.float64)
    assert _load().oracle_gconv_bwd_data(ctypes.byref(d), _ptr(dy), _ptr(w), _ptr(dx), int(nthreads)) == 0
    return dx


def bwd_filter(x, dy, *, K, stride=1, pad=0, groups, O, layout=NCHW, nthreads=1):
    x = _f64(x); dy = _f64(dy)
    d, yshape, wshape = _shapes(x.shape, K, stride, pad, groups, O, layout)
    assert dy.shape == yshape, (dy.shape, yshape)
    dw = np.empty(wshape, dtype=np.float64)
    assert _load().oracle_gconv_bwd_filter(ctypes.byref(d), _ptr(x), _ptr(dy), _ptr(dw), int(nthreads)) == 0
    return dw


# ---- second route: dense product with a group mask (NCHW, numpy, builds the big matrices) ----------

def group_mask(C, O, K, groups):
    """0/1 matrix [O, C*K*K]: ones where output channel o and input channel c share a group."""
    Cg, Og = C // groups, O // groups
    A = np.zeros((O, C * K * K), dtype=np.float64)
    for o in range(O):
        g = o // Og
        A[o, g * Cg * K * K:(g + 1) * Cg * K * K] = 1.0
    return A


def dense_weights(w, C, K, groups):
    """The full [O, C*K*K] weight matrix with w [O,Cg,K,K] placed in the blocks of its group."""
    w = np.asarray(w, dtype=np.float64)
    O, Cg = w.shape[0], w.shape[1]
    Og = O // groups
    Wd = np.zeros((O, C * K * K), dtype=np.float64)
    for o in range(O):
        g = o // Og
        Wd[o, g * Cg * K * K:(g + 1) * Cg * K * K] = w[o].reshape(-1)
    return Wd


def dense_group_fwd(x, w, K, stride, pad, groups):
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    O = w.shape[0]
    What = dense_weights(w, C, K, groups) * group_mask(C, O, K, groups)
    out = []
    for n in range(N):
        cols, Ho, Wo = im2col(x[n], K, stride, pad)
        out.append((What @ cols).reshape(O, Ho, Wo))
    return np.stack(out)


def dense_group_bwd_data(dy, w, x_shape, K, stride, pad, groups):
    dy = np.asarray(dy, dtype=np.float64)
    N, C, H, W = x_shape
    O = w.shape[0]
    What = dense_weights(w, C, K, groups) * group_mask(C, O, K, groups)
    dx = np.empty(x_shape, dtype=np.float64)
    for n in range(N):
        dx[n] = col2im(What.T @ dy[n].reshape(O, -1), C, H, W, K, stride, pad)
    return dx


def dense_group_bwd_filter(x, dy, K, stride, pad, groups):
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    N, C, H, W = x.shape
    O = dy.shape[1]
    Cg, Og = C // groups, O // groups
    g = np.zeros((O, C * K * K), dtype=np.float64)
    for n in range(N):
        cols, Ho, Wo = im2col(x[n], K, stride, pad)
        g += dy[n].reshape(O, -1) @ cols.T
    g *= group_mask(C, O, K, groups)
    dw = np.empty((O, Cg, K, K), dtype=np.float64)
    for o in range(O):
        gi = o // Og
        dw[o] = g[o, gi * Cg * K * K:(gi + 1) * Cg * K * K].reshape(Cg, K, K)
    return dw
