"""Helpers shared by the GPU parity tests: run the three passes through the C ABI and compare
with the CPU oracle under the stated tolerances."""
import numpy as np
import torch

import oracle
import paper_1803_09926_amd as dw
from paper_1803_09926_amd import workloads as wl

# Tolerances (relative error, both as max|g-r|/max|r| and as ||g-r||_2/||r||_2):
# fp32 forward and backward-data 1e-5, fp32 backward-filter 1e-4, bf16 storage 1e-2.
TOL_F32 = 1e-5
TOL_F32_FILTER = 1e-4
TOL_BF16 = 1e-2


def rel_errors(got, ref):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    diff = got - ref
    denom_max = max(np.abs(ref).max(), 1e-300)
    denom_l2 = max(np.sqrt((ref * ref).sum()), 1e-300)
    return np.abs(diff).max() / denom_max, np.sqrt((diff * diff).sum()) / denom_l2


def assert_close(got, ref, tol, what):
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), what + ": non-finite output"
    if np.abs(ref).max() == 0.0:
        assert np.abs(got).max() == 0.0, what
        return
    emax, el2 = rel_errors(got, ref)
    assert emax <= tol and el2 <= tol, "%s: max-norm rel err %.3e, l2 rel err %.3e, tol %.1e" % (what, emax, el2, tol)


def to_dev(a_f32: np.ndarray, dtype: int):
    t = torch.from_numpy(np.ascontiguousarray(a_f32)).cuda()
    return t if dtype == wl.F32 else t.to(torch.bfloat16)     # exact: values are already bf16-representable


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def desc_for(layer, N, layout, dtype):
    return dw.desc(N, layer.C, layer.H, layer.W, layer.K, layer.stride, layer.pad, layer.mult, layout, dtype)


def shapes(layer, N, layout):
    if layout == wl.NCHW:
        return (N, layer.C, layer.H, layer.W), (N, layer.O, layer.Ho, layer.Wo), (layer.O, layer.K, layer.K)
    return (N, layer.H, layer.W, layer.C), (N, layer.Ho, layer.Wo, layer.O), (layer.K, layer.K, layer.O)


def gpu_passes(layer, N, layout, dtype, xt, wt, dyt, stream=None, poison=True):
    """Run fwd, bwd_data, bwd_filter on device tensors; outputs are pre-filled with NaN so an
    unwritten element cannot pass."""
    d = desc_for(layer, N, layout, dtype)
    xs, ys, ws = shapes(layer, N, layout)
    tdt = torch.float32 if dtype == wl.F32 else torch.bfloat16
    fill = float("nan") if poison else 0.0
    y = torch.full(ys, fill, device="cuda", dtype=tdt)
    dx = torch.full(xs, fill, device="cuda", dtype=tdt)
    dwt = torch.full(ws, fill, device="cuda", dtype=torch.float32)
    wsb = torch.full((max(dw.bwd_filter_workspace_bytes(d), 16),), 0xFF, device="cuda", dtype=torch.uint8)
    dw.fwd(d, xt, wt, y, stream)
    dw.bwd_data(d, dyt, wt, dx, stream)
    dw.bwd_filter(d, xt, dyt, dwt, wsb, stream)
    torch.cuda.synchronize()
    return y, dx, dwt


def gpu_bwd(layer, N, layout, dtype, xt, wt, dyt, stream=None):
    """The whole backward pass through dwconv_bwd (fused where a fused kernel exists); outputs pre-filled with NaN."""
    d = desc_for(layer, N, layout, dtype)
    xs, ys, ws = shapes(layer, N, layout)
    tdt = torch.float32 if dtype == wl.F32 else torch.bfloat16
    dx = torch.full(xs, float("nan"), device="cuda", dtype=tdt)
    dwt = torch.full(ws, float("nan"), device="cuda", dtype=torch.float32)
    wsb = torch.full((max(dw.bwd_workspace_bytes(d), 16),), 0xFF, device="cuda", dtype=torch.uint8)
    dw.bwd(d, xt, dyt, wt, dx, dwt, wsb, stream)
    torch.cuda.synchronize()
    return dx, dwt


def check_layer_full(layer, N, layout, dtype, seed):
    """Whole-tensor, element-by-element comparison with the oracle (small problems)."""
    x, w, dy = wl.make_inputs(layer, N, layout, dtype, seed)
    y, dx, dwt = gpu_passes(layer, N, layout, dtype, to_dev(x, dtype), to_dev(w, dtype), to_dev(dy, dtype))
    kw = dict(K=layer.K, stride=layer.stride, pad=layer.pad, mult=layer.mult, layout=layout, nthreads=8)
    tol = TOL_F32 if dtype == wl.F32 else TOL_BF16
    tolf = TOL_F32_FILTER
    tag = "%s N=%d layout=%d dtype=%d" % (layer.name, N, layout, dtype)
    assert_close(to_host(y), oracle.fwd(x, w, **kw), tol, "fwd " + tag)
    assert_close(to_host(dx), oracle.bwd_data(dy, w, x_shape=x.shape, **kw), tol, "bwd_data " + tag)
    ref_dx = oracle.bwd_data(dy, w, x_shape=x.shape, **kw)
    ref_dw = oracle.bwd_filter(x, dy, **kw)
    assert_close(to_host(dwt), ref_dw, tolf, "bwd_filter " + tag)
    dx2, dw2 = gpu_bwd(layer, N, layout, dtype, to_dev(x, dtype), to_dev(w, dtype), to_dev(dy, dtype))
    assert_close(to_host(dx2), ref_dx, tol, "bwd (dx) " + tag)
    assert_close(to_host(dw2), ref_dw, tolf, "bwd (dw) " + tag)
