"""The entry point that allocates nothing (dwconv_bwd_filter_noalloc) against dwconv_bwd_filter: same kernels, the
partial sums in the library's fixed device array instead of a workspace.  Two calls in a row, the second on a smaller
input, so that what the first call left in the array would show if it were ever read."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_1803_09926_amd as dw
from paper_1803_09926_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu

# (layer, batch): a large first call (many partials), then a smaller one; several kernel families
SEQUENCES = [
    ("nhwc_f32", wl.NHWC, wl.F32, [(wl.Layer("big", 64, 56, 56), 16), (wl.Layer("small", 24, 14, 14), 3)]),
    ("nchw_f32", wl.NCHW, wl.F32, [(wl.Layer("big", 48, 28, 28), 12), (wl.Layer("small", 8, 14, 14), 2)]),
    ("nchw_bf16_s2", wl.NCHW, wl.BF16, [(wl.Layer("big", 32, 32, 32, 3, 2, 1), 8), (wl.Layer("small", 8, 16, 16, 3, 2, 1), 2)]),
    ("nhwc_bf16_k5", wl.NHWC, wl.BF16, [(wl.Layer("big", 32, 28, 28, 5, 1, 2), 8), (wl.Layer("small", 6, 9, 11, 5, 1, 2), 1)]),
    ("generic", wl.NCHW, wl.F32, [(wl.Layer("big", 10, 19, 23, 7, 3, 2), 5), (wl.Layer("small", 3, 9, 5, 4, 1, 0), 2)]),
]


@pytest.mark.parametrize("name,layout,dtype,seq", SEQUENCES, ids=[s[0] for s in SEQUENCES])
def test_noalloc_filter_gradient_matches_the_workspace_entry_point(name, layout, dtype, seq):
    tdt = torch.float32 if dtype == wl.F32 else torch.bfloat16
    for step, (layer, N) in enumerate(seq):
        print("noalloc", name, "call", step, layer, "N", N, flush=True)
        x, w, dy = wl.make_inputs(layer, N, layout, dtype, seed=700 + step)
        xt, dyt = (torch.from_numpy(a).cuda().to(tdt) for a in (x, dy))
        d = dw.desc(N, layer.C, layer.H, layer.W, layer.K, layer.stride, layer.pad, layer.mult, layout, dtype)
        need = dw.bwd_filter_workspace_bytes(d)
        assert 0 < need <= 16 << 20
        ws = torch.empty(need, device="cuda", dtype=torch.uint8)
        want = torch.full(w.shape, float("nan"), device="cuda", dtype=torch.float32)
        got = torch.full(w.shape, float("nan"), device="cuda", dtype=torch.float32)
        dw.bwd_filter(d, xt, dyt, want, ws)
        dw.bwd_filter_noalloc(d, xt, dyt, got)
        torch.cuda.synchronize()
        # same kernels, same order of additions: bit for bit
        assert torch.equal(got, want), (name, step)
        ref = oracle.bwd_filter(x, dy, K=layer.K, stride=layer.stride, pad=layer.pad, mult=layer.mult, layout=layout)
        gu.assert_close(gu.to_host(got), ref, gu.TOL_F32_FILTER, "noalloc bwd_filter %s call %d" % (name, step))


def test_noalloc_rejects_shapes_beyond_its_scratch_and_bad_arguments():
    lib = dw.load()
    # very many channels: 18 MiB of partial sums, beyond the 16 MiB array (nothing is launched for it)
    big = dw.desc(1, 262144, 7, 7, 3, 1, 1, 1, wl.NHWC, wl.F32)
    assert dw.bwd_filter_workspace_bytes(big) > 16 << 20
    a = torch.zeros(64, device="cuda")
    p = ctypes.c_void_p(a.data_ptr())
    assert lib.dwconv_bwd_filter_noalloc(ctypes.byref(big), p, p, p, None) == -9
    assert "scratch" in dw.status_string(-9)
    ok = dw.desc(2, 8, 16, 16)
    assert lib.dwconv_bwd_filter_noalloc(ctypes.byref(ok), None, p, p, None) == -1
    assert lib.dwconv_bwd_filter_noalloc(ctypes.byref(ok), p, p, ctypes.c_void_p(a.data_ptr() + 4), None) == -5
    bad = dw.desc(2, 0, 16, 16)
    assert lib.dwconv_bwd_filter_noalloc(ctypes.byref(bad), p, p, p, None) == -2
