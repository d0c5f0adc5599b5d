"""Brute-force second route to the depthwise results: the paper's own identity.

TEST INFRASTRUCTURE ONLY (used to pin the loop-nest oracle on tiny inputs).

Paper Section II ("standard convolutions"): a standard convolution is an im2col
step, X (M x F x F) -> C ((M*K*K) x (F*F)) with every K x K block a column, and a
dense product Z = W C with W of shape N_out x (M*K*K).  Section III-A, Eq. 1-3:
a depthwise convolution equals that standard convolution when the per-channel
filters w(i) are placed on the block diagonal of W and every other entry is 0
(W_hat = W (.) A with A the 0/1 block-diagonal mask of Eq. 2).  Eq. 4: the
depthwise weight gradient is the dense weight gradient masked by A.
Section III-B: splitting the channels into G groups and refactorising each group
on its own gives the same result.

Everything here is NCHW, fp64, numpy, and deliberately builds the big matrices.
Channel multiplier m (not in the paper, which has m = 1): output channel o reads
input channel o // m, so row o of W_hat is non-zero only in column block o // m.
"""
from __future__ import annotations

import numpy as np


def im2col(x_img, K, stride, pad):
    """x_img [M,H,W] -> C [(M*K*K), (Ho*Wo)]; row index (ch*K + kh)*K + kw."""
    M, H, W = x_img.shape
    Ho = (H + 2 * pad - K) // stride + 1
    Wo = (W + 2 * pad - K) // stride + 1
    xp = np.zeros((M, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    xp[:, pad:pad + H, pad:pad + W] = x_img
    cols = np.empty((M * K * K, Ho * Wo), dtype=np.float64)
    for ch in range(M):
        for kh in range(K):
            for kw in range(K):
                patch = xp[ch, kh:kh + stride * (Ho - 1) + 1:stride, kw:kw + stride * (Wo - 1) + 1:stride]
                cols[(ch * K + kh) * K + kw] = patch.reshape(-1)
    return cols, Ho, Wo


def col2im(dcols, M, H, W, K, stride, pad):
    """Transpose of im2col: scatter-add columns back onto a [M,H,W] map."""
    Ho = (H + 2 * pad - K) // stride + 1
    Wo = (W + 2 * pad - K) // stride + 1
    dxp = np.zeros((M, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    for ch in range(M):
        for kh in range(K):
            for kw in range(K):
                dxp[ch, kh:kh + stride * (Ho - 1) + 1:stride, kw:kw + stride * (Wo - 1) + 1:stride] += \
                    dcols[(ch * K + kh) * K + kw].reshape(Ho, Wo)
    return dxp[:, pad:pad + H, pad:pad + W]


def mask(M, K, mult=1):
    """A of Eq. 2, shape [M*mult, M*K*K]: ones in block (o, o // mult)."""
    A = np.zeros((M * mult, M * K * K), dtype=np.float64)
    for o in range(M * mult):
        c = o // mult
        A[o, c * K * K:(c + 1) * K * K] = 1.0
    return A


def refactorize(w, M, K, mult=1):
    """W of Eq. 1: the filter vectors w [O,K,K] on the block diagonal, zeros elsewhere."""
    O = M * mult
    Wd = np.zeros((O, M * K * K), dtype=np.float64)
    for o in range(O):
        c = o // mult
        Wd[o, c * K * K:(c + 1) * K * K] = np.asarray(w[o], dtype=np.float64).reshape(-1)
    return Wd


def _groups(M, G):
    assert M % G == 0
    size = M // G
    return [(g * size, (g + 1) * size) for g in range(G)]


def fwd(x, w, K, stride, pad, mult=1, G=1):
    """Z = W_hat (x) X per image, group by group.  x [N,M,H,W], w [M*mult,K,K]."""
    x = np.asarray(x, dtype=np.float64)
    N, M, H, W = x.shape
    out = None
    for n in range(N):
        rows = []
        for c0, c1 in _groups(M, G):
            Mg = c1 - c0
            wg = w[c0 * mult:c1 * mult]
            What = refactorize(wg, Mg, K, mult) * mask(Mg, K, mult)
            cols, Ho, Wo = im2col(x[n, c0:c1], K, stride, pad)
            rows.append(What @ cols)
        Z = np.concatenate(rows, axis=0).reshape(M * mult, Ho, Wo)
        if out is None:
            out = np.empty((N,) + Z.shape, dtype=np.float64)
        out[n] = Z
    return out


def bwd_data(dy, w, x_shape, K, stride, pad, mult=1, G=1):
    """dC = W_hat^T dZ, then col2im."""
    dy = np.asarray(dy, dtype=np.float64)
    N, M, H, W = x_shape
    dx = np.empty(x_shape, dtype=np.float64)
    for n in range(N):
        for c0, c1 in _groups(M, G):
            Mg = c1 - c0
            What = refactorize(w[c0 * mult:c1 * mult], Mg, K, mult) * mask(Mg, K, mult)
            dZ = dy[n, c0 * mult:c1 * mult].reshape(Mg * mult, -1)
            dx[n, c0:c1] = col2im(What.T @ dZ, Mg, H, W, K, stride, pad)
    return dx


def dense_weight_grad(x, dy, K, stride, pad, mult=1):
    """The unmasked dense gradient dW_hat = sum_n dZ_n C_n^T, shape [M*mult, M*K*K]."""
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    N, M, H, W = x.shape
    O = M * mult
    g = np.zeros((O, M * K * K), dtype=np.float64)
    for n in range(N):
        cols, Ho, Wo = im2col(x[n], K, stride, pad)
        g += dy[n].reshape(O, -1) @ cols.T
    return g


def bwd_filter(x, dy, K, stride, pad, mult=1):
    """Eq. 4: mask the dense gradient, then read the diagonal blocks back as [O,K,K]."""
    N, M, H, W = x.shape
    O = M * mult
    g = dense_weight_grad(x, dy, K, stride, pad, mult) * mask(M, K, mult)
    dw = np.empty((O, K, K), dtype=np.float64)
    for o in range(O):
        c = o // mult
        dw[o] = g[o, c * K * K:(c + 1) * K * K].reshape(K, K)
    return dw
