"""Pins for the CPU oracle: everything here is independent of the oracle's own loop nests.

Routes used: the paper's block-diagonal dense-convolution identity (Section III-A, Eq. 1-4) and
its grouped form (Section III-B) as brute force; hand-derived all-ones closed forms
(tests/golden); adjoint and bilinearity identities; exact finite differences (the loss
sum(dy*y) is linear in x and in w); special cases that reduce to a per-channel scale, a
subsampling, a dot product, or the forward pass with a rotated filter; layout equivalence;
and, as one more library cross-check, torch's grouped conv2d with autograd on the CPU.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import dense_identity as dense

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "all_ones_closed_forms.txt")


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def odim(i, K, s, p):
    return (i + 2 * p - K) // s + 1


TINY = [
    # N, C, H, W, K, s, p, m
    (2, 4, 5, 5, 3, 1, 1, 1),
    (1, 6, 7, 6, 3, 2, 1, 1),
    (2, 3, 6, 7, 3, 2, 0, 1),
    (1, 4, 7, 7, 5, 1, 2, 1),
    (1, 2, 7, 5, 5, 2, 2, 2),
    (2, 6, 4, 4, 1, 1, 0, 1),
    (1, 3, 7, 7, 3, 3, 1, 3),
    (1, 2, 5, 6, 3, 1, 2, 2),   # pad larger than needed: rows of pure zeros
    (1, 2, 2, 2, 3, 1, 1, 1),   # map smaller than the filter
    (1, 4, 6, 6, 2, 2, 0, 1),   # even kernel
]


def divisors(c):
    return [g for g in range(1, c + 1) if c % g == 0]


@pytest.mark.parametrize("N,C,H,W,K,s,p,m", TINY)
def test_fwd_equals_block_diagonal_dense_convolution(N, C, H, W, K, s, p, m):
    x = rnd((N, C, H, W), 1); w = rnd((C * m, K, K), 2)
    y = oracle.fwd(x, w, K=K, stride=s, pad=p, mult=m)
    for G in divisors(C):
        yd = dense.fwd(x, w, K, s, p, m, G)
        np.testing.assert_allclose(y, yd, rtol=0, atol=1e-12)


@pytest.mark.parametrize("N,C,H,W,K,s,p,m", TINY)
def test_bwd_data_equals_transposed_dense_convolution(N, C, H, W, K, s, p, m):
    dy = rnd((N, C * m, odim(H, K, s, p), odim(W, K, s, p)), 3); w = rnd((C * m, K, K), 4)
    dx = oracle.bwd_data(dy, w, x_shape=(N, C, H, W), K=K, stride=s, pad=p, mult=m)
    for G in divisors(C):
        dxd = dense.bwd_data(dy, w, (N, C, H, W), K, s, p, m, G)
        np.testing.assert_allclose(dx, dxd, rtol=0, atol=1e-12)


@pytest.mark.parametrize("N,C,H,W,K,s,p,m", TINY)
def test_bwd_filter_equals_masked_dense_gradient(N, C, H, W, K, s, p, m):
    x = rnd((N, C, H, W), 5); dy = rnd((N, C * m, odim(H, K, s, p), odim(W, K, s, p)), 6)
    dw = oracle.bwd_filter(x, dy, K=K, stride=s, pad=p, mult=m)
    np.testing.assert_allclose(dw, dense.bwd_filter(x, dy, K, s, p, m), rtol=0, atol=1e-11)
    if C > 1:
        # the mask is doing work: the dense gradient has non-zero off-diagonal entries
        g = dense.dense_weight_grad(x, dy, K, s, p, m)
        off = g * (1.0 - dense.mask(C, K, m))
        assert np.abs(off).max() > 1e-3


def _golden():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, vals = line.split(":")
            toks = head.split()
            kind = toks[0]
            kv = dict(t.split("=") for t in toks[1:])
            cases.append((kind, {k: int(v) for k, v in kv.items()}, [float(v) for v in vals.split()]))
    return cases


@pytest.mark.parametrize("kind,kv,vals", _golden())
def test_all_ones_golden(kind, kv, vals):
    K, s, p, H, W = kv["K"], kv["s"], kv["p"], kv["H"], kv["W"]
    N = kv.get("N", 1)
    C = 2
    Ho, Wo = odim(H, K, s, p), odim(W, K, s, p)
    for layout in (oracle.NCHW, oracle.NHWC):
        xs = (N, C, H, W) if layout == oracle.NCHW else (N, H, W, C)
        ys = (N, C, Ho, Wo) if layout == oracle.NCHW else (N, Ho, Wo, C)
        ws = (C, K, K) if layout == oracle.NCHW else (K, K, C)
        if kind == "fwd":
            y = oracle.fwd(np.ones(xs), np.ones(ws), K=K, stride=s, pad=p, layout=layout)
            got = y[0, 1] if layout == oracle.NCHW else y[0, :, :, 1]
        elif kind == "bwd_data":
            dx = oracle.bwd_data(np.ones(ys), np.ones(ws), x_shape=xs, K=K, stride=s, pad=p, layout=layout)
            got = dx[0, 1] if layout == oracle.NCHW else dx[0, :, :, 1]
        else:
            dw = oracle.bwd_filter(np.ones(xs), np.ones(ys), K=K, stride=s, pad=p, layout=layout)
            got = dw[1] if layout == oracle.NCHW else dw[:, :, 1]
        np.testing.assert_array_equal(got.reshape(-1), np.array(vals))


def count_T(o, dim, K, s, p):
    return sum(1 for k in range(K) if 0 <= o * s - p + k < dim)


def count_U(i, dim, out, K, s, p):
    return sum(1 for k in range(K) if (i + p - k) % s == 0 and 0 <= (i + p - k) // s < out)


def count_R(k, dim, out, K, s, p):
    return sum(1 for o in range(out) if 0 <= o * s - p + k < dim)


@pytest.mark.parametrize("H,W,K,s,p,m", [(9, 7, 3, 1, 1, 1), (8, 11, 3, 2, 1, 2), (7, 7, 5, 1, 2, 1),
                                         (10, 9, 5, 2, 2, 3), (6, 6, 3, 3, 0, 1), (5, 8, 4, 2, 1, 1)])
def test_all_ones_counting_formulas(H, W, K, s, p, m):
    N, C = 3, 2
    Ho, Wo = odim(H, K, s, p), odim(W, K, s, p)
    O = C * m
    y = oracle.fwd(np.ones((N, C, H, W)), np.ones((O, K, K)), K=K, stride=s, pad=p, mult=m)
    T = np.outer([count_T(o, H, K, s, p) for o in range(Ho)], [count_T(o, W, K, s, p) for o in range(Wo)])
    np.testing.assert_array_equal(y, np.broadcast_to(T, y.shape))
    dx = oracle.bwd_data(np.ones((N, O, Ho, Wo)), np.ones((O, K, K)), x_shape=(N, C, H, W), K=K, stride=s, pad=p, mult=m)
    U = m * np.outer([count_U(i, H, Ho, K, s, p) for i in range(H)], [count_U(i, W, Wo, K, s, p) for i in range(W)])
    np.testing.assert_array_equal(dx, np.broadcast_to(U, dx.shape))
    dw = oracle.bwd_filter(np.ones((N, C, H, W)), np.ones((N, O, Ho, Wo)), K=K, stride=s, pad=p, mult=m)
    R = N * np.outer([count_R(k, H, Ho, K, s, p) for k in range(K)], [count_R(k, W, Wo, K, s, p) for k in range(K)])
    np.testing.assert_array_equal(dw, np.broadcast_to(R, dw.shape))
    # the three counts tally the same set of (output pixel, tap) pairs
    assert T.sum() == R.sum() // N == U.sum() // m


SHAPES = [(2, 5, 9, 8, 3, 1, 1, 1), (2, 4, 9, 10, 3, 2, 1, 1), (1, 3, 11, 9, 5, 1, 2, 2),
          (2, 2, 8, 8, 5, 2, 2, 1), (1, 4, 7, 7, 3, 1, 1, 3), (1, 3, 9, 9, 3, 4, 1, 1), (2, 3, 6, 5, 2, 1, 1, 2)]


@pytest.mark.parametrize("layout", [oracle.NCHW, oracle.NHWC])
@pytest.mark.parametrize("N,C,H,W,K,s,p,m", SHAPES)
def test_adjoint_and_bilinear_identities(N, C, H, W, K, s, p, m, layout):
    O, Ho, Wo = C * m, odim(H, K, s, p), odim(W, K, s, p)
    xs = (N, C, H, W) if layout == oracle.NCHW else (N, H, W, C)
    ys = (N, O, Ho, Wo) if layout == oracle.NCHW else (N, Ho, Wo, O)
    ws = (O, K, K) if layout == oracle.NCHW else (K, K, O)
    x, w, dy = rnd(xs, 7), rnd(ws, 8), rnd(ys, 9)
    kw = dict(K=K, stride=s, pad=p, mult=m, layout=layout)
    L = np.sum(dy * oracle.fwd(x, w, **kw))
    dx = oracle.bwd_data(dy, w, x_shape=xs, **kw)
    dw = oracle.bwd_filter(x, dy, **kw)
    assert abs(L - np.sum(dx * x)) <= 1e-11 * max(1.0, abs(L))     # <dy, fwd(x)> = <bwd_data(dy), x>
    assert abs(L - np.sum(dw * w)) <= 1e-11 * max(1.0, abs(L))     # <dy, fwd(x; w)> = <bwd_filter(x,dy), w>


@pytest.mark.parametrize("N,C,H,W,K,s,p,m", SHAPES[:5])
def test_exact_finite_differences(N, C, H, W, K, s, p, m):
    O, Ho, Wo = C * m, odim(H, K, s, p), odim(W, K, s, p)
    x, w, dy = rnd((N, C, H, W), 10), rnd((O, K, K), 11), rnd((N, O, Ho, Wo), 12)
    kw = dict(K=K, stride=s, pad=p, mult=m)
    L0 = np.sum(dy * oracle.fwd(x, w, **kw))
    dx = oracle.bwd_data(dy, w, x_shape=x.shape, **kw)
    dw = oracle.bwd_filter(x, dy, **kw)
    rng = np.random.default_rng(13)
    for _ in range(12):       # the loss is linear in x: a unit step gives the derivative exactly
        idx = tuple(rng.integers(0, d) for d in x.shape)
        xp = x.copy(); xp[idx] += 1.0
        assert abs(np.sum(dy * oracle.fwd(xp, w, **kw)) - L0 - dx[idx]) < 1e-10
    for idx in itertools.product(range(O), range(K), range(K)):     # and linear in w: every entry
        wp = w.copy(); wp[idx] += 1.0
        assert abs(np.sum(dy * oracle.fwd(x, wp, **kw)) - L0 - dw[idx]) < 1e-10


def test_k1_is_a_per_channel_scale_and_dot_product():
    N, C, H, W, m = 2, 3, 5, 4, 2
    x, w, dy = rnd((N, C, H, W), 14), rnd((C * m, 1, 1), 15), rnd((N, C * m, H, W), 16)
    y = oracle.fwd(x, w, K=1, mult=m)
    xr = np.repeat(x, m, axis=1)
    np.testing.assert_allclose(y, xr * w.reshape(1, -1, 1, 1), rtol=0, atol=1e-14)
    dw = oracle.bwd_filter(x, dy, K=1, mult=m)
    np.testing.assert_allclose(dw.reshape(-1), np.einsum("nohw,nohw->o", xr, dy), rtol=0, atol=1e-12)
    dx = oracle.bwd_data(dy, w, x_shape=x.shape, K=1, mult=m)
    np.testing.assert_allclose(dx, (dy * w.reshape(1, -1, 1, 1)).reshape(N, C, m, H, W).sum(2), rtol=0, atol=1e-13)


@pytest.mark.parametrize("K,s", [(3, 1), (3, 2), (5, 1), (5, 3)])
def test_delta_filter_subsamples_and_zero_stuffs(K, s):
    N, C, H, W = 2, 3, 9, 8
    p = K // 2
    x = rnd((N, C, H, W), 17)
    w = np.zeros((C, K, K)); w[:, p, p] = 1.0
    y = oracle.fwd(x, w, K=K, stride=s, pad=p)
    np.testing.assert_array_equal(y, x[:, :, ::s, ::s])
    dy = rnd(y.shape, 18)
    dx = oracle.bwd_data(dy, w, x_shape=x.shape, K=K, stride=s, pad=p)
    up = np.zeros_like(x); up[:, :, ::s, ::s] = dy
    np.testing.assert_array_equal(dx, up)


def test_off_centre_delta_filter_pins_the_shift_direction():
    # w[o,0,2] = 1 (top-right tap), 3x3 pad 1: y[oh,ow] = x[oh-1, ow+1]: cross-correlation, no flip
    x = rnd((1, 1, 5, 6), 19)
    w = np.zeros((1, 3, 3)); w[0, 0, 2] = 1.0
    y = oracle.fwd(x, w, K=3, stride=1, pad=1)
    exp = np.zeros_like(x); exp[0, 0, 1:, :-1] = x[0, 0, :-1, 1:]
    np.testing.assert_array_equal(y, exp)


@pytest.mark.parametrize("K,p,m", [(3, 1, 1), (5, 2, 1), (3, 0, 2), (5, 1, 3)])
def test_stride1_bwd_data_is_fwd_with_rotated_filter(K, p, m):
    N, C, H, W = 2, 3, 8, 9
    O, Ho, Wo = C * m, odim(H, K, 1, p), odim(W, K, 1, p)
    dy, w = rnd((N, O, Ho, Wo), 20), rnd((O, K, K), 21)
    dx = oracle.bwd_data(dy, w, x_shape=(N, C, H, W), K=K, stride=1, pad=p, mult=m)
    rot = w[:, ::-1, ::-1]
    acc = np.zeros((N, C, H, W))
    for q in range(m):
        acc += oracle.fwd(dy[:, q::m], rot[q::m], K=K, stride=1, pad=K - 1 - p)
    np.testing.assert_allclose(dx, acc, rtol=0, atol=1e-12)


@pytest.mark.parametrize("N,C,H,W,K,s,p,m", SHAPES)
def test_nhwc_equals_nchw_after_transposition(N, C, H, W, K, s, p, m):
    O, Ho, Wo = C * m, odim(H, K, s, p), odim(W, K, s, p)
    x, w, dy = rnd((N, C, H, W), 22), rnd((O, K, K), 23), rnd((N, O, Ho, Wo), 24)
    kw = dict(K=K, stride=s, pad=p, mult=m)
    t = lambda a: np.ascontiguousarray(a.transpose(0, 2, 3, 1))
    tw = lambda a: np.ascontiguousarray(a.transpose(1, 2, 0))
    np.testing.assert_array_equal(t(oracle.fwd(x, w, **kw)), oracle.fwd(t(x), tw(w), layout=oracle.NHWC, **kw))
    np.testing.assert_allclose(t(oracle.bwd_data(dy, w, x_shape=x.shape, **kw)),
                               oracle.bwd_data(t(dy), tw(w), x_shape=t(x).shape, layout=oracle.NHWC, **kw),
                               rtol=0, atol=1e-13)
    np.testing.assert_allclose(tw(oracle.bwd_filter(x, dy, **kw)),
                               oracle.bwd_filter(t(x), t(dy), layout=oracle.NHWC, **kw), rtol=0, atol=1e-13)


def test_linearity_and_interior_translation():
    N, C, H, W, K = 1, 2, 10, 10, 3
    x1, x2, w = rnd((N, C, H, W), 25), rnd((N, C, H, W), 26), rnd((C, K, K), 27)
    f = lambda x: oracle.fwd(x, w, K=K, stride=1, pad=1)
    np.testing.assert_allclose(f(2.0 * x1 - 3.0 * x2), 2.0 * f(x1) - 3.0 * f(x2), rtol=0, atol=1e-12)
    xs = np.zeros_like(x1); xs[:, :, 2:, 1:] = x1[:, :, :-2, :-1]
    np.testing.assert_allclose(f(xs)[:, :, 3:-1, 2:-1], f(x1)[:, :, 1:-3, 1:-2], rtol=0, atol=1e-13)


def test_threads_do_not_change_the_result():
    x, w, dy = rnd((4, 6, 9, 9), 28), rnd((6, 3, 3), 29), rnd((4, 6, 5, 5), 30)
    kw = dict(K=3, stride=2, pad=1)
    np.testing.assert_array_equal(oracle.fwd(x, w, **kw), oracle.fwd(x, w, nthreads=4, **kw))
    np.testing.assert_array_equal(oracle.bwd_data(dy, w, x_shape=x.shape, **kw),
                                  oracle.bwd_data(dy, w, x_shape=x.shape, nthreads=4, **kw))
    np.testing.assert_array_equal(oracle.bwd_filter(x, dy, **kw), oracle.bwd_filter(x, dy, nthreads=4, **kw))


@pytest.mark.parametrize("N,C,H,W,K,s,p,m", SHAPES)
def test_against_torch_grouped_conv2d_cpu(N, C, H, W, K, s, p, m):
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    O, Ho, Wo = C * m, odim(H, K, s, p), odim(W, K, s, p)
    x, w, dy = rnd((N, C, H, W), 31), rnd((O, K, K), 32), rnd((N, O, Ho, Wo), 33)
    xt = torch.tensor(x, requires_grad=True); wt = torch.tensor(w.reshape(O, 1, K, K), requires_grad=True)
    yt = F.conv2d(xt, wt, stride=s, padding=p, groups=C)
    yt.backward(torch.tensor(dy))
    kw = dict(K=K, stride=s, pad=p, mult=m)
    np.testing.assert_allclose(oracle.fwd(x, w, **kw), yt.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.bwd_data(dy, w, x_shape=x.shape, **kw), xt.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.bwd_filter(x, dy, **kw), wt.grad.numpy().reshape(O, K, K), rtol=0, atol=1e-11)
