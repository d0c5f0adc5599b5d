"""The paper's own route (Section III-A, Eq. 1-4, with the grouping of Section III-B) as built for the on-box
comparison, checked element by element against the CPU oracle: the dense forward product, the dense input gradient
(transposed product and col2im) and the masked dense weight gradient have to be the depthwise layer's three passes.
The oracle is the reference, not this library: the comparison leg must be right in its own right before its timings
mean anything.  Runs on the CPU with torch's CPU operators, and on the GPU machine with the library GEMMs it times."""
import numpy as np
import pytest
import torch

import oracle
from paper_1803_09926_amd import workloads as wl
from paper_1803_09926_amd.dense_comparison import DenseRoute

import gpu_util as gu

# two tiny layers: stride 1 with two group sizes, and a stride-2 layer on an odd-sized map
CASES = [
    ("k3s1", 3, wl.Layer("dense_k3s1", 8, 9, 11, 3, 1, 1), (2, 4, 8)),
    ("k3s2", 2, wl.Layer("dense_k3s2", 6, 10, 7, 3, 2, 1), (2, 3, 6)),
    ("k5s1", 2, wl.Layer("dense_k5s1", 4, 8, 8, 5, 1, 2), (1, 4)),
]


def _check(device):
    for name, N, layer, sizes in CASES:
        x, w, dy = wl.make_inputs(layer, N, wl.NCHW, wl.F32, seed=4242)
        kw = dict(K=layer.K, stride=layer.stride, pad=layer.pad, mult=1, layout=wl.NCHW)
        ref_y = oracle.fwd(x, w, **kw)
        ref_dx = oracle.bwd_data(dy, w, x_shape=x.shape, **kw)
        ref_dw = oracle.bwd_filter(x, dy, **kw)
        xt, wt, dyt = (torch.from_numpy(a).to(device) for a in (x, w, dy))
        for S in sizes:
            route = DenseRoute(wt, N, layer.C, layer.H, layer.W, layer.K, layer.stride, layer.pad, S)
            z = route.fwd(xt)
            gx, gw = route.bwd(dyt)
            tag = "%s S=%d on %s" % (name, S, device)
            gu.assert_close(z.cpu().numpy(), ref_y, gu.TOL_F32, "dense route fwd " + tag)
            gu.assert_close(gx.cpu().numpy(), ref_dx, gu.TOL_F32, "dense route bwd_data " + tag)
            gu.assert_close(route.filter_gradient(gw).cpu().numpy(), ref_dw, gu.TOL_F32_FILTER,
                            "dense route bwd_filter " + tag)
            # Eq. 4's mask does work: everything outside the diagonal blocks is exactly zero after it, and the
            # unmasked dense gradient is not
            KK = layer.K * layer.K
            blocks = gw.view(route.G, S, S, KK).cpu().numpy()
            off = [blocks[:, i, j] for i in range(S) for j in range(S) if i != j]
            assert all(np.all(b == 0.0) for b in off), tag


def test_dense_route_matches_the_oracle_on_cpu():
    _check("cpu")


@pytest.mark.gpu
def test_dense_route_matches_the_oracle_on_gpu():
    _check("cuda")
