"""MI355X-native depthwise-convolution training kernels (forward, backward-data, backward-filter).

Thin binding over the C ABI in include/dwconv.h: argument marshalling only.  Every step of the
computation runs in the HIP kernels of libdwconv.so; there is no CPU or PyTorch fallback, and
`load()` raises if the library has not been built.  PyTorch supplies device memory and streams.
"""
from __future__ import annotations

import contextlib
import ctypes
import os

NCHW = 0
NHWC = 1
F32 = 0
BF16 = 1

PASS_FWD, PASS_BWD_DATA, PASS_BWD_FILTER = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdwconv.so")
_lib = None

EXPORTS = ("dwconv_out_dims", "dwconv_bwd_filter_workspace_bytes", "dwconv_fwd", "dwconv_bwd_data",
           "dwconv_bwd_filter", "dwconv_bwd_workspace_bytes", "dwconv_bwd", "dwconv_status_string",
           "dwconv_variant_name", "dwconv_tuning_reload", "dwconv_bwd_filter_noalloc",
           "gconv_out_dims", "gconv_bwd_filter_workspace_bytes", "gconv_fwd", "gconv_bwd_data", "gconv_bwd_filter",
           "gconv_variant_name")


class Desc(ctypes.Structure):
    """Mirror of struct dwconv_desc."""
    _fields_ = [(k, ctypes.c_int32) for k in
                ("N", "C", "H", "W", "K", "stride", "pad", "mult", "layout", "dtype")]


class GroupDesc(ctypes.Structure):
    """Mirror of struct dwconv_group_desc."""
    _fields_ = [(k, ctypes.c_int32) for k in
                ("N", "C", "H", "W", "K", "stride", "pad", "groups", "O", "layout", "dtype")]


class DwconvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


def load():
    """Load libdwconv.so; raise if it is missing (the product has no other code path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libdwconv.so is not built: run `python -m paper_1803_09926_amd.build` "
                           "(or __graft_entry__.build()) first; there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    P, VP, I32P = ctypes.POINTER(Desc), ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
    lib.dwconv_out_dims.argtypes = [P, I32P, I32P]; lib.dwconv_out_dims.restype = ctypes.c_int
    lib.dwconv_bwd_filter_workspace_bytes.argtypes = [P]; lib.dwconv_bwd_filter_workspace_bytes.restype = ctypes.c_size_t
    lib.dwconv_fwd.argtypes = [P, VP, VP, VP, VP]; lib.dwconv_fwd.restype = ctypes.c_int
    lib.dwconv_bwd_data.argtypes = [P, VP, VP, VP, VP]; lib.dwconv_bwd_data.restype = ctypes.c_int
    lib.dwconv_bwd_filter.argtypes = [P, VP, VP, VP, VP, ctypes.c_size_t, VP]; lib.dwconv_bwd_filter.restype = ctypes.c_int
    lib.dwconv_bwd_workspace_bytes.argtypes = [P]; lib.dwconv_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.dwconv_bwd.argtypes = [P, VP, VP, VP, VP, VP, VP, ctypes.c_size_t, VP]; lib.dwconv_bwd.restype = ctypes.c_int
    lib.dwconv_status_string.argtypes = [ctypes.c_int]; lib.dwconv_status_string.restype = ctypes.c_char_p
    lib.dwconv_variant_name.argtypes = [P, ctypes.c_int]; lib.dwconv_variant_name.restype = ctypes.c_char_p
    lib.dwconv_bwd_filter_noalloc.argtypes = [P, VP, VP, VP, VP]; lib.dwconv_bwd_filter_noalloc.restype = ctypes.c_int
    lib.dwconv_tuning_reload.argtypes = []; lib.dwconv_tuning_reload.restype = ctypes.c_int
    G = ctypes.POINTER(GroupDesc)
    lib.gconv_out_dims.argtypes = [G, I32P, I32P]; lib.gconv_out_dims.restype = ctypes.c_int
    lib.gconv_bwd_filter_workspace_bytes.argtypes = [G]; lib.gconv_bwd_filter_workspace_bytes.restype = ctypes.c_size_t
    lib.gconv_fwd.argtypes = [G, VP, VP, VP, VP]; lib.gconv_fwd.restype = ctypes.c_int
    lib.gconv_bwd_data.argtypes = [G, VP, VP, VP, VP]; lib.gconv_bwd_data.restype = ctypes.c_int
    lib.gconv_bwd_filter.argtypes = [G, VP, VP, VP, VP, ctypes.c_size_t, VP]; lib.gconv_bwd_filter.restype = ctypes.c_int
    lib.gconv_variant_name.argtypes = [G, ctypes.c_int]; lib.gconv_variant_name.restype = ctypes.c_char_p
    _lib = lib
    return lib


def desc(N, C, H, W, K=3, stride=1, pad=1, mult=1, layout=NCHW, dtype=F32) -> Desc:
    return Desc(int(N), int(C), int(H), int(W), int(K), int(stride), int(pad), int(mult), int(layout), int(dtype))


def status_string(status: int) -> str:
    return load().dwconv_status_string(int(status)).decode()


def variant_name(d: Desc, which: int) -> str:
    return load().dwconv_variant_name(ctypes.byref(d), int(which)).decode()


def tuning_reload() -> int:
    """Take a new snapshot of the DWCONV_TUNE_* environment variables (tuning sweeps and forced-tiling tests only;
    holds nothing unless DWCONV_TUNE=1 is set).  Returns the number of variables in the snapshot."""
    return int(load().dwconv_tuning_reload())


@contextlib.contextmanager
def tuning_overrides(knobs: dict):
    """Run a block with the given DWCONV_TUNE_* variables in force (tuning sweeps and forced-tiling tests): sets them and
    the master switch, takes a snapshot, and on exit restores the environment and takes the snapshot again."""
    names = list(knobs) + ["DWCONV_TUNE"]
    saved = {k: os.environ.get(k) for k in names}
    try:
        for k, v in knobs.items():
            os.environ[k] = str(v)
        os.environ["DWCONV_TUNE"] = "1"
        tuning_reload()
        yield
    finally:
        for k, v in saved.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
        tuning_reload()


def out_dims(d: Desc):
    ho, wo = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = load().dwconv_out_dims(ctypes.byref(d), ctypes.byref(ho), ctypes.byref(wo))
    if rc != 0:
        raise DwconvError(rc, "dwconv_out_dims")
    return ho.value, wo.value


def bwd_filter_workspace_bytes(d: Desc) -> int:
    return int(load().dwconv_bwd_filter_workspace_bytes(ctypes.byref(d)))


def bwd_workspace_bytes(d: Desc) -> int:
    return int(load().dwconv_bwd_workspace_bytes(ctypes.byref(d)))


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check_tensor(t, name, d: Desc, numel: int, fp32_always=False):
    import torch
    want = torch.float32 if (fp32_always or d.dtype == F32) else torch.bfloat16
    if not t.is_cuda:
        raise ValueError("%s must be a device tensor" % name)
    if t.dtype != want:
        raise ValueError("%s must be %s" % (name, want))
    if not t.is_contiguous() or t.numel() != numel:
        raise ValueError("%s must be contiguous with %d elements (has %d)" % (name, numel, t.numel()))


def _sizes(d: Desc):
    ho, wo = out_dims(d)
    O = d.C * d.mult
    return d.N * d.C * d.H * d.W, d.N * O * ho * wo, O * d.K * d.K


def fwd(d: Desc, x, w, y, stream=None):
    """Enqueue y = depthwise cross-correlation of x with w on `stream` (default: torch's current)."""
    nx, ny, nw = _sizes(d)
    _check_tensor(x, "x", d, nx); _check_tensor(w, "w", d, nw); _check_tensor(y, "y", d, ny)
    rc = load().dwconv_fwd(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(y), _stream(stream))
    if rc != 0:
        raise DwconvError(rc, "dwconv_fwd")
    return y


def bwd_data(d: Desc, dy, w, dx, stream=None):
    """Enqueue dx = input gradient."""
    nx, ny, nw = _sizes(d)
    _check_tensor(dy, "dy", d, ny); _check_tensor(w, "w", d, nw); _check_tensor(dx, "dx", d, nx)
    rc = load().dwconv_bwd_data(ctypes.byref(d), _ptr(dy), _ptr(w), _ptr(dx), _stream(stream))
    if rc != 0:
        raise DwconvError(rc, "dwconv_bwd_data")
    return dx


def bwd_filter(d: Desc, x, dy, dw, workspace, stream=None):
    """Enqueue dw = filter gradient (fp32).  `workspace` is a uint8 device tensor of at least
    bwd_filter_workspace_bytes(d) bytes."""
    nx, ny, nw = _sizes(d)
    _check_tensor(x, "x", d, nx); _check_tensor(dy, "dy", d, ny); _check_tensor(dw, "dw", d, nw, fp32_always=True)
    if workspace is None or not workspace.is_cuda:
        raise ValueError("workspace must be a device tensor")
    nbytes = workspace.numel() * workspace.element_size()
    rc = load().dwconv_bwd_filter(ctypes.byref(d), _ptr(x), _ptr(dy), _ptr(dw), _ptr(workspace),
                                  ctypes.c_size_t(nbytes), _stream(stream))
    if rc != 0:
        raise DwconvError(rc, "dwconv_bwd_filter")
    return dw


def bwd_filter_noalloc(d: Desc, x, dy, dw, stream=None):
    """Enqueue dw = filter gradient (fp32) through the entry point that allocates nothing and takes no workspace
    (the partial sums go to a fixed array inside the library; shapes that need more raise DWCONV_ERR_SCRATCH)."""
    nx, ny, nw = _sizes(d)
    _check_tensor(x, "x", d, nx); _check_tensor(dy, "dy", d, ny); _check_tensor(dw, "dw", d, nw, fp32_always=True)
    rc = load().dwconv_bwd_filter_noalloc(ctypes.byref(d), _ptr(x), _ptr(dy), _ptr(dw), _stream(stream))
    if rc != 0:
        raise DwconvError(rc, "dwconv_bwd_filter_noalloc")
    return dw


def bwd(d: Desc, x, dy, w, dx, dw, workspace, stream=None):
    """Enqueue the whole backward pass: dx = input gradient, dw = filter gradient (fp32).  `workspace` is a
    uint8 device tensor of at least bwd_workspace_bytes(d) bytes."""
    nx, ny, nw = _sizes(d)
    _check_tensor(x, "x", d, nx); _check_tensor(dy, "dy", d, ny); _check_tensor(w, "w", d, nw)
    _check_tensor(dx, "dx", d, nx); _check_tensor(dw, "dw", d, nw, fp32_always=True)
    if workspace is None or not workspace.is_cuda:
        raise ValueError("workspace must be a device tensor")
    nbytes = workspace.numel() * workspace.element_size()
    rc = load().dwconv_bwd(ctypes.byref(d), _ptr(x), _ptr(dy), _ptr(w), _ptr(dx), _ptr(dw), _ptr(workspace),
                           ctypes.c_size_t(nbytes), _stream(stream))
    if rc != 0:
        raise DwconvError(rc, "dwconv_bwd")
    return dx, dw


# ---- group convolution (more than one channel per group) ----------------------------------------------

def group_desc(N, C, H, W, K=3, stride=1, pad=1, groups=1, O=None, layout=NCHW, dtype=F32) -> GroupDesc:
    return GroupDesc(int(N), int(C), int(H), int(W), int(K), int(stride), int(pad), int(groups),
                     int(C if O is None else O), int(layout), int(dtype))


def gconv_variant_name(d: GroupDesc, which: int) -> str:
    return load().gconv_variant_name(ctypes.byref(d), int(which)).decode()


def gconv_out_dims(d: GroupDesc):
    ho, wo = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = load().gconv_out_dims(ctypes.byref(d), ctypes.byref(ho), ctypes.byref(wo))
    if rc != 0:
        raise DwconvError(rc, "gconv_out_dims")
    return ho.value, wo.value


def gconv_bwd_filter_workspace_bytes(d: GroupDesc) -> int:
    return int(load().gconv_bwd_filter_workspace_bytes(ctypes.byref(d)))


def _gsizes(d: GroupDesc):
    ho, wo = gconv_out_dims(d)
    return d.N * d.C * d.H * d.W, d.N * d.O * ho * wo, d.O * (d.C // d.groups) * d.K * d.K


def gconv_fwd(d: GroupDesc, x, w, y, stream=None):
    """Enqueue y = group cross-correlation of x with w (w [O,Cg,K,K] for NCHW, [K,K,Cg,O] for NHWC)."""
    nx, ny, nw = _gsizes(d)
    _check_tensor(x, "x", d, nx); _check_tensor(w, "w", d, nw); _check_tensor(y, "y", d, ny)
    rc = load().gconv_fwd(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(y), _stream(stream))
    if rc != 0:
        raise DwconvError(rc, "gconv_fwd")
    return y


def gconv_bwd_data(d: GroupDesc, dy, w, dx, stream=None):
    """Enqueue dx = input gradient of the group convolution."""
    nx, ny, nw = _gsizes(d)
    _check_tensor(dy, "dy", d, ny); _check_tensor(w, "w", d, nw); _check_tensor(dx, "dx", d, nx)
    rc = load().gconv_bwd_data(ctypes.byref(d), _ptr(dy), _ptr(w), _ptr(dx), _stream(stream))
    if rc != 0:
        raise DwconvError(rc, "gconv_bwd_data")
    return dx


def gconv_bwd_filter(d: GroupDesc, x, dy, dw, workspace, stream=None):
    """Enqueue dw = filter gradient (fp32) of the group convolution.  `workspace` is a uint8 device tensor of
    at least gconv_bwd_filter_workspace_bytes(d) bytes."""
    nx, ny, nw = _gsizes(d)
    _check_tensor(x, "x", d, nx); _check_tensor(dy, "dy", d, ny); _check_tensor(dw, "dw", d, nw, fp32_always=True)
    if workspace is None or not workspace.is_cuda:
        raise ValueError("workspace must be a device tensor")
    nbytes = workspace.numel() * workspace.element_size()
    rc = load().gconv_bwd_filter(ctypes.byref(d), _ptr(x), _ptr(dy), _ptr(dw), _ptr(workspace),
                                 ctypes.c_size_t(nbytes), _stream(stream))
    if rc != 0:
        raise DwconvError(rc, "gconv_bwd_filter")
    return dw
