"""On-box comparison with the paper's own route: diagonalwise refactorization with grouping.

COMPARISON ONLY, never a code path of the library.  For every depthwise layer of MobileNet-v1 (the shapes of
the paper's Table III) this times

  * this library's kernels through the C ABI (forward; backward = backward-filter + backward-data), and
  * the refactorised dense route of Section III: the channels are split into groups of S (Section III-B,
    grouping "by size"), each group's filters are placed on the block diagonal of an S x (S*K*K) matrix
    (Eq. 1), the input is unrolled with im2col (Section II) and the two are multiplied with a plain batched
    GEMM (torch.matmul, i.e. rocBLAS / hipBLASLt); backward = the two transposed GEMMs, col2im, and the mask
    of Eq. 4 on the weight gradient.  There is no cuDNN analogue here and none is claimed: the point is the
    S-fold redundant arithmetic and the 9-fold im2col traffic on this chip, i.e. the shape of the paper's
    Fig. 5 (time against group size).

Usage:  python -m paper_1803_09926_amd.dense_comparison [--batch 64] [--sizes 16,32,64,128] [--iters 5]
Prints one table row per layer and a JSON line with the totals.
"""
from __future__ import annotations

import argparse
import json
import sys


class DenseRoute:
    """The refactorised layer of Section III for one group size S, on NCHW fp32 device tensors.

    Eq. 1: the S filters of a group sit on the block diagonal of an S x (S*K*K) matrix; Eq. 2: the 0/1 mask of the
    same shape; forward = im2col (Section II) and one batched GEMM per group; backward = the two transposed GEMMs,
    col2im, and the mask of Eq. 4 on the dense weight gradient."""

    def __init__(self, w, N, C, H, W, K, stride, pad, S):
        import torch
        assert C % S == 0
        self.N, self.C, self.H, self.W, self.K, self.s, self.p, self.S, self.G = N, C, H, W, K, stride, pad, S, C // S
        self.Ho, self.Wo = (H + 2 * pad - K) // stride + 1, (W + 2 * pad - K) // stride + 1
        G, KK = self.G, K * K
        self.What = torch.zeros(G, S, S * KK, device=w.device)
        self.A = torch.zeros(S, S * KK, device=w.device)
        wv = w.reshape(G, S, KK)
        for i in range(S):
            self.What[:, i, i * KK:(i + 1) * KK] = wv[:, i]
            self.A[i, i * KK:(i + 1) * KK] = 1.0
        self.cols = None

    def fwd(self, x):
        import torch
        import torch.nn.functional as F
        N, G, S, K = self.N, self.G, self.S, self.K
        L = self.Ho * self.Wo
        self.cols = F.unfold(x.view(N * G, S, self.H, self.W), K, padding=self.p, stride=self.s).view(N, G, S * K * K, L)
        return torch.matmul(self.What.unsqueeze(0), self.cols).view(N, self.C, self.Ho, self.Wo)

    def bwd(self, dy):
        """Input gradient [N,C,H,W] and the masked dense weight gradient [G,S,S*K*K] (needs the im2col matrix that
        fwd left behind, as a training step has it)."""
        import torch
        import torch.nn.functional as F
        N, G, S, K = self.N, self.G, self.S, self.K
        L = self.Ho * self.Wo
        dz = dy.view(N, G, S, L)
        dcols = torch.matmul(self.What.transpose(1, 2).unsqueeze(0), dz)
        gx = F.fold(dcols.view(N * G, S * K * K, L), (self.H, self.W), K, padding=self.p, stride=self.s)
        gw = torch.matmul(dz, self.cols.transpose(2, 3)).sum(0) * self.A.unsqueeze(0)        # Eq. 4
        return gx.view(N, self.C, self.H, self.W), gw

    def filter_gradient(self, gw):
        """The per-channel filter gradient [C,K,K]: the diagonal blocks of the masked dense gradient."""
        import torch
        G, S, KK = self.G, self.S, self.K * self.K
        blocks = gw.view(G, S, S, KK)
        idx = torch.arange(S, device=gw.device)
        return blocks[:, idx, idx, :].reshape(self.C, self.K, self.K)


def _time(fn, torch, iters):
    fn(); fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--sizes", default="16,32,64,128")
    ap.add_argument("--iters", type=int, default=5)
    args = ap.parse_args()
    import torch
    import paper_1803_09926_amd as dw
    from paper_1803_09926_amd import workloads as wl
    if not torch.cuda.is_available():
        sys.exit("dense_comparison needs a GPU")
    dw.load()
    N = args.batch
    sizes = [int(s) for s in args.sizes.split(",")]
    print("%-28s %9s %9s | %s" % ("layer (batch %d, fp32 NCHW)" % N, "ours fwd", "ours bwd",
                                  "  ".join("S=%-4d fwd / bwd ms" % s for s in sizes)))
    tot = {"ours_fwd": 0.0, "ours_bwd": 0.0}
    for li, layer in enumerate(wl.MOBILENET_V1):
        x, w, dy = wl.make_inputs_device(layer, N, wl.NCHW, wl.F32, seed=li)
        C, H, W, K, s, p = layer.C, layer.H, layer.W, layer.K, layer.stride, layer.pad
        Ho, Wo, L = layer.Ho, layer.Wo, layer.Ho * layer.Wo
        d = dw.desc(N, C, H, W, K, s, p, 1, wl.NCHW, wl.F32)
        y = torch.empty_like(dy); dx = torch.empty_like(x); dwt = torch.empty_like(w)
        ws = torch.empty(max(dw.bwd_filter_workspace_bytes(d), 16), device="cuda", dtype=torch.uint8)
        t_f = _time(lambda: dw.fwd(d, x, w, y), torch, args.iters)
        t_b = _time(lambda: (dw.bwd_filter(d, x, dy, dwt, ws), dw.bwd_data(d, dy, w, dx)), torch, args.iters)
        tot["ours_fwd"] += t_f; tot["ours_bwd"] += t_b
        cells = []
        for S in sizes:
            if C % S != 0:
                cells.append("%-22s" % "-")
                continue
            route = DenseRoute(w, N, C, H, W, K, s, p, S)
            fwd = lambda: route.fwd(x)
            bwd = lambda: route.bwd(dy)
            z = fwd()
            dw.fwd(d, x, w, y)
            torch.cuda.synchronize()
            err = float((z - y).abs().max() / y.abs().max())
            assert err < 1e-4, (layer.name, S, err)      # the two routes compute the same layer
            gx, gw = bwd()
            dw.bwd_data(d, dy, w, dx)
            torch.cuda.synchronize()
            assert float((gx - dx).abs().max() / dx.abs().max()) < 1e-4, (layer.name, S)
            td_f = _time(fwd, torch, args.iters)
            td_b = _time(bwd, torch, args.iters)
            tot.setdefault("dense_fwd_S%d" % S, 0.0); tot.setdefault("dense_bwd_S%d" % S, 0.0)
            tot["dense_fwd_S%d" % S] += td_f; tot["dense_bwd_S%d" % S] += td_b
            cells.append("%8.3f / %-11.3f" % (td_f, td_b))
            del route, z, gx, gw
            torch.cuda.empty_cache()
        print("%-28s %9.4f %9.4f | %s" % (layer.name[10:], t_f, t_b, "  ".join(cells)), flush=True)
    print(json.dumps({"batch": N, "unit": "ms, sum over the 13 layers (a dense total covers only the layers whose "
                      "channel count the group size divides)", **{k: round(v, 3) for k, v in tot.items()}}))


if __name__ == "__main__":
    main()
