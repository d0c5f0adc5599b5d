"""CPU oracle for depthwise-convolution training (forward, backward-data, backward-filter).

TEST INFRASTRUCTURE ONLY: the slow fp64 checker the GPU library is compared with.
Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the GPU package never does, and this package never imports it.

The arithmetic lives in ``dwconv_oracle.c`` (plain loop nests that write out the
definition of a depthwise convolution, paper Section II and Section III-A, Eq. 3
and Eq. 4).  This module only compiles that file with gcc and marshals numpy
arrays into it.  ``dense_identity`` holds a second, separately written route to
the same results (the paper's block-diagonal dense convolution), used to pin
the loop nests on tiny inputs.  ``gconv`` is the oracle of the group-convolution
extension (more than one channel per group), with its own C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dwconv_oracle.c")
_LIB = os.path.join(_HERE, "libdwconv_oracle.so")
_lock = threading.Lock()
_lib = None

NCHW = 0
NHWC = 1


class _Desc(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in
                ("N", "C", "H", "W", "K", "stride", "pad", "mult", "layout")]


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc -O2, OpenMP for the optional outer-loop split)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            dp = ctypes.POINTER(ctypes.c_double)
            for name in ("oracle_dwconv_fwd", "oracle_dwconv_bwd_data", "oracle_dwconv_bwd_filter"):
                fn = getattr(lib, name)
                fn.argtypes = [ctypes.POINTER(_Desc), dp, dp, dp, ctypes.c_int]
                fn.restype = ctypes.c_int
            lib.oracle_out_dims.argtypes = [ctypes.POINTER(_Desc), ctypes.POINTER(ctypes.c_int32),
                                            ctypes.POINTER(ctypes.c_int32)]
            lib.oracle_out_dims.restype = ctypes.c_int
            lib.oracle_threads_available.restype = ctypes.c_int
            _lib = lib
    return _lib


def threads_available() -> int:
    return int(_load().oracle_threads_available())


def _desc(N, C, H, W, K, stride, pad, mult, layout):
    return _Desc(int(N), int(C), int(H), int(W), int(K), int(stride), int(pad), int(mult), int(layout))


def out_dims(H, W, K, stride, pad):
    d = _desc(1, 1, H, W, K, stride, pad, 1, 0)
    ho, wo = ctypes.c_int32(0), ctypes.c_int32(0)
    if _load().oracle_out_dims(ctypes.byref(d), ctypes.byref(ho), ctypes.byref(wo)):
        raise ValueError("invalid depthwise-convolution shape")
    return ho.value, wo.value


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _shapes(x_shape, K, stride, pad, mult, layout):
    if layout == NCHW:
        N, C, H, W = x_shape
    else:
        N, H, W, C = x_shape
    Ho, Wo = out_dims(H, W, K, stride, pad)
    O = C * mult
    yshape = (N, O, Ho, Wo) if layout == NCHW else (N, Ho, Wo, O)
    wshape = (O, K, K) if layout == NCHW else (K, K, O)
    return N, C, H, W, O, Ho, Wo, yshape, wshape


def fwd(x, w, *, K, stride=1, pad=0, mult=1, layout=NCHW, nthreads=1):
    """y = depthwise cross-correlation of x with w.  Returns fp64."""
    x = _f64(x); w = _f64(w)
    N, C, H, W, O, Ho, Wo, yshape, wshape = _shapes(x.shape, K, stride, pad, mult, layout)
    assert w.shape == wshape, (w.shape, wshape)
    y = np.empty(yshape, dtype=np.float64)
    d = _desc(N, C, H, W, K, stride, pad, mult, layout)
    rc = _load().oracle_dwconv_fwd(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(y), int(nthreads))
    assert rc == 0
    return y


def bwd_data(dy, w, *, x_shape, K, stride=1, pad=0, mult=1, layout=NCHW, nthreads=1):
    """dx = gradient of sum(dy * fwd(x, w)) with respect to x.  Returns fp64."""
    dy = _f64(dy); w = _f64(w)
    N, C, H, W, O, Ho, Wo, yshape, wshape = _shapes(tuple(x_shape), K, stride, pad, mult, layout)
    assert dy.shape == yshape, (dy.shape, yshape)
    assert w.shape == wshape, (w.shape, wshape)
    dx = np.empty(tuple(x_shape), dtype=np.float64)
    d = _desc(N, C, H, W, K, stride, pad, mult, layout)
    rc = _load().oracle_dwconv_bwd_data(ctypes.byref(d), _ptr(dy), _ptr(w), _ptr(dx), int(nthreads))
    assert rc == 0
    return dx


def bwd_filter(x, dy, *, K, stride=1, pad=0, mult=1, layout=NCHW, nthreads=1):
    """dw = gradient of sum(dy * fwd(x, w)) with respect to w (summed over the batch).  Returns fp64."""
    x = _f64(x); dy = _f64(dy)
    N, C, H, W, O, Ho, Wo, yshape, wshape = _shapes(x.shape, K, stride, pad, mult, layout)
    assert dy.shape == yshape, (dy.shape, yshape)
    dw = np.empty(wshape, dtype=np.float64)
    d = _desc(N, C, H, W, K, stride, pad, mult, layout)
    rc = _load().oracle_dwconv_bwd_filter(ctypes.byref(d), _ptr(x), _ptr(dy), _ptr(dw), int(nthreads))
    assert rc == 0
    return dw
