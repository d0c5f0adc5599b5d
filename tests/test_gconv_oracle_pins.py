"""Pins for the group-convolution CPU oracle, all independent of its loop nests.

Routes: the dense im2col product with the weight matrix masked group-wise (the mask of the paper's
Section III-A, Eq. 2, generalised as Section V-B describes: a block per pair of channels of the same
group) as brute force; the depthwise oracle (pinned on its own) for groups == C; adjoint identities
(the loss sum(dy*y) is bilinear in x and w); all-ones closed forms; a one-hot filter entry that pins
which input channel and which shift an entry (o, ci, kh, kw) stands for; layout equivalence; torch's
grouped conv2d with autograd on the CPU as a library cross-check.  At the end, planted mistakes
(textual mutants of the C file) that at least one of these pins has to catch.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle
from oracle import gconv

SRC = os.path.join(os.path.dirname(gconv.__file__), "gconv_oracle.c")


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def odim(i, K, s, p):
    return (i + 2 * p - K) // s + 1


TINY = [
    # N, C, O, G, H, W, K, s, p
    (2, 4, 4, 2, 5, 5, 3, 1, 1),
    (1, 6, 9, 3, 7, 6, 3, 2, 1),
    (2, 8, 4, 2, 6, 7, 3, 2, 0),
    (1, 4, 8, 1, 7, 7, 5, 1, 2),     # one group: a standard convolution
    (1, 6, 6, 6, 5, 6, 3, 1, 1),     # as many groups as channels: depthwise
    (1, 3, 6, 3, 5, 5, 3, 1, 1),     # depthwise with channel multiplier 2
    (2, 6, 2, 2, 4, 4, 1, 1, 0),
    (1, 4, 4, 2, 2, 2, 3, 1, 1),     # map smaller than the filter
    (1, 8, 8, 2, 6, 6, 2, 2, 0),     # even kernel, four channels per group
]


def _inputs(N, C, O, G, H, W, K, s, p, seed=0):
    x = rnd((N, C, H, W), seed + 1)
    w = rnd((O, C // G, K, K), seed + 2)
    dy = rnd((N, O, odim(H, K, s, p), odim(W, K, s, p)), seed + 3)
    return x, w, dy


@pytest.mark.parametrize("N,C,O,G,H,W,K,s,p", TINY)
def test_fwd_equals_group_masked_dense_convolution(N, C, O, G, H, W, K, s, p):
    x, w, _ = _inputs(N, C, O, G, H, W, K, s, p)
    y = gconv.fwd(x, w, K=K, stride=s, pad=p, groups=G, O=O)
    np.testing.assert_allclose(y, gconv.dense_group_fwd(x, w, K, s, p, G), rtol=0, atol=1e-11)


@pytest.mark.parametrize("N,C,O,G,H,W,K,s,p", TINY)
def test_bwd_data_equals_transposed_masked_dense_convolution(N, C, O, G, H, W, K, s, p):
    x, w, dy = _inputs(N, C, O, G, H, W, K, s, p)
    dx = gconv.bwd_data(dy, w, x_shape=x.shape, K=K, stride=s, pad=p, groups=G, O=O)
    np.testing.assert_allclose(dx, gconv.dense_group_bwd_data(dy, w, x.shape, K, s, p, G), rtol=0, atol=1e-11)


@pytest.mark.parametrize("N,C,O,G,H,W,K,s,p", TINY)
def test_bwd_filter_equals_masked_dense_gradient(N, C, O, G, H, W, K, s, p):
    x, w, dy = _inputs(N, C, O, G, H, W, K, s, p)
    dw = gconv.bwd_filter(x, dy, K=K, stride=s, pad=p, groups=G, O=O)
    np.testing.assert_allclose(dw, gconv.dense_group_bwd_filter(x, dy, K, s, p, G), rtol=0, atol=1e-10)


@pytest.mark.parametrize("C,m,K,s,p", [(5, 1, 3, 1, 1), (4, 2, 3, 2, 1), (3, 3, 5, 1, 2)])
def test_as_many_groups_as_channels_is_the_depthwise_layer(C, m, K, s, p):
    N, H, W = 2, 7, 6
    O = C * m
    x = rnd((N, C, H, W), 11); w = rnd((O, K, K), 12); dy = rnd((N, O, odim(H, K, s, p), odim(W, K, s, p)), 13)
    kw = dict(K=K, stride=s, pad=p, groups=C, O=O)
    np.testing.assert_allclose(gconv.fwd(x, w[:, None], **kw), oracle.fwd(x, w, K=K, stride=s, pad=p, mult=m), atol=1e-12)
    np.testing.assert_allclose(gconv.bwd_data(dy, w[:, None], x_shape=x.shape, **kw),
                               oracle.bwd_data(dy, w, x_shape=x.shape, K=K, stride=s, pad=p, mult=m), atol=1e-12)
    np.testing.assert_allclose(gconv.bwd_filter(x, dy, **kw)[:, 0],
                               oracle.bwd_filter(x, dy, K=K, stride=s, pad=p, mult=m), atol=1e-11)


@pytest.mark.parametrize("N,C,O,G,H,W,K,s,p", TINY)
def test_adjoint_identities(N, C, O, G, H, W, K, s, p):
    x, w, dy = _inputs(N, C, O, G, H, W, K, s, p, seed=20)
    kw = dict(K=K, stride=s, pad=p, groups=G, O=O)
    loss = float(np.sum(dy * gconv.fwd(x, w, **kw)))
    assert abs(loss - float(np.sum(gconv.bwd_data(dy, w, x_shape=x.shape, **kw) * x))) <= 1e-9 * max(1.0, abs(loss))
    assert abs(loss - float(np.sum(gconv.bwd_filter(x, dy, **kw) * w))) <= 1e-9 * max(1.0, abs(loss))


def test_all_ones_closed_forms():
    # 3x3, stride 1, pad 1 on ones: an output counts Cg * (taps inside the image); the filter
    # gradient of tap (kh,kw) counts N * (output pixels whose tap is inside), for every (o, ci)
    N, C, O, G, H, W = 2, 6, 4, 2, 4, 5
    Cg = C // G
    x = np.ones((N, C, H, W)); w = np.ones((O, Cg, 3, 3)); dy = np.ones((N, O, H, W))
    y = gconv.fwd(x, w, K=3, stride=1, pad=1, groups=G, O=O)
    rows = np.array([2] + [3] * (H - 2) + [2]); cols = np.array([2] + [3] * (W - 2) + [2])
    np.testing.assert_array_equal(y, np.broadcast_to(Cg * np.outer(rows, cols), y.shape))
    dx = gconv.bwd_data(dy, w, x_shape=x.shape, K=3, stride=1, pad=1, groups=G, O=O)
    np.testing.assert_array_equal(dx, np.broadcast_to((O // G) * np.outer(rows, cols), dx.shape))
    dw = gconv.bwd_filter(x, dy, K=3, stride=1, pad=1, groups=G, O=O)
    cnt_h = np.array([H - 1, H, H - 1]); cnt_w = np.array([W - 1, W, W - 1])
    np.testing.assert_array_equal(dw, np.broadcast_to(N * np.outer(cnt_h, cnt_w), dw.shape))


def test_one_hot_filter_entry_pins_channel_and_shift():
    # w[o, ci, kh, kw] = 1 alone: y[o] is x[channel (o // Og) * Cg + ci] shifted by (kh - p, kw - p)
    N, C, O, G, H, W, K, p = 1, 6, 4, 2, 5, 6, 3, 1
    Cg, Og = C // G, O // G
    x = rnd((N, C, H, W), 30)
    for o, ci, kh, kw in [(0, 2, 0, 1), (3, 1, 2, 0), (2, 0, 1, 2)]:
        w = np.zeros((O, Cg, K, K)); w[o, ci, kh, kw] = 1.0
        y = gconv.fwd(x, w, K=K, stride=1, pad=p, groups=G, O=O)
        src = x[0, (o // Og) * Cg + ci]
        want = np.zeros((H, W))
        for oh in range(H):
            for ow in range(W):
                ih, iw = oh - p + kh, ow - p + kw
                if 0 <= ih < H and 0 <= iw < W:
                    want[oh, ow] = src[ih, iw]
        np.testing.assert_array_equal(y[0, o], want)
        others = [q for q in range(O) if q != o]
        assert np.all(y[0, others] == 0.0)


@pytest.mark.parametrize("N,C,O,G,H,W,K,s,p", TINY[:4])
def test_nhwc_is_nchw_transposed(N, C, O, G, H, W, K, s, p):
    x, w, dy = _inputs(N, C, O, G, H, W, K, s, p, seed=40)
    kw = dict(K=K, stride=s, pad=p, groups=G, O=O)
    xl, dyl = x.transpose(0, 2, 3, 1), dy.transpose(0, 2, 3, 1)
    wl = w.transpose(2, 3, 1, 0)      # [K,K,Cg,O]
    y = gconv.fwd(xl, wl, layout=gconv.NHWC, **kw)
    np.testing.assert_allclose(y.transpose(0, 3, 1, 2), gconv.fwd(x, w, **kw), atol=1e-12)
    dx = gconv.bwd_data(dyl, wl, x_shape=xl.shape, layout=gconv.NHWC, **kw)
    np.testing.assert_allclose(dx.transpose(0, 3, 1, 2), gconv.bwd_data(dy, w, x_shape=x.shape, **kw), atol=1e-12)
    dw = gconv.bwd_filter(xl, dyl, layout=gconv.NHWC, **kw)
    np.testing.assert_allclose(dw.transpose(3, 2, 0, 1), gconv.bwd_filter(x, dy, **kw), atol=1e-11)


@pytest.mark.parametrize("N,C,O,G,H,W,K,s,p", TINY)
def test_against_torch_grouped_conv2d(N, C, O, G, H, W, K, s, p):
    import torch
    x, w, dy = _inputs(N, C, O, G, H, W, K, s, p, seed=50)
    xt = torch.tensor(x, requires_grad=True); wt = torch.tensor(w, requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wt, stride=s, padding=p, groups=G)
    yt.backward(torch.tensor(dy))
    kw = dict(K=K, stride=s, pad=p, groups=G, O=O)
    np.testing.assert_allclose(gconv.fwd(x, w, **kw), yt.detach().numpy(), atol=1e-11)
    np.testing.assert_allclose(gconv.bwd_data(dy, w, x_shape=x.shape, **kw), xt.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(gconv.bwd_filter(x, dy, **kw), wt.grad.numpy(), atol=1e-10)


def test_rejects_channel_counts_the_groups_do_not_divide():
    with pytest.raises(ValueError):
        gconv.fwd(np.zeros((1, 5, 4, 4)), np.zeros((4, 2, 3, 3)), K=3, stride=1, pad=1, groups=2, O=4)
    with pytest.raises(ValueError):
        gconv.fwd(np.zeros((1, 4, 4, 4)), np.zeros((3, 2, 3, 3)), K=3, stride=1, pad=1, groups=2, O=3)


# ---- planted mistakes --------------------------------------------------------------------------

MUTANTS = [
    ("fwd_wrong_group_base", "const int c0 = (o / Og) * Cg; /* first input channel of the group of o */", "const int c0 = (o / Cg) * Og;", None),
    ("fwd_filter_flipped", "acc += w[wat(L, O, Cg, K, o, ci, kh, kw)] * x[", "acc += w[wat(L, O, Cg, K, o, ci, K - 1 - kh, K - 1 - kw)] * x[", None),
    ("fwd_channel_order_reversed", "x[at(L, C, H, W, n, c0 + ci, ih, iw)];\n                            }\n                    y[", "x[at(L, C, H, W, n, c0 + Cg - 1 - ci, ih, iw)];\n                            }\n                    y[", None),
    ("bwd_data_pad_sign", "int ih = oh * s - p + kh, iw = ow * s - p + kw;", "int ih = oh * s + p - kh, iw = ow * s + p - kw;", 1),
    ("bwd_data_drops_a_channel", "for (int ci = 0; ci < Cg; ++ci)\n                        for (int kh = 0; kh < K; ++kh)\n                            for (int kw = 0; kw < K; ++kw) {\n                                int ih = oh * s - p + kh, iw = ow * s - p + kw;\n                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;\n                                dx[", "for (int ci = 0; ci < Cg - (Cg > 1); ++ci)\n                        for (int kh = 0; kh < K; ++kh)\n                            for (int kw = 0; kw < K; ++kw) {\n                                int ih = oh * s - p + kh, iw = ow * s - p + kw;\n                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;\n                                dx[", None),
    ("bwd_filter_taps_transposed", "dw[wat(L, O, Cg, K, o, ci, kh, kw)] = acc;", "dw[wat(L, O, Cg, K, o, ci, kw, kh)] = acc;", None),
    ("bwd_filter_mean_over_batch", "dw[wat(L, O, Cg, K, o, ci, kh, kw)] = acc;", "dw[wat(L, O, Cg, K, o, ci, kh, kw)] = acc / N;", None),
    ("nhwc_filter_layout", "return (((size_t)kh * K + kw) * Cg + ci) * O + o;", "return (((size_t)kh * K + kw) * O + o) * Cg + ci;", None),
    ("nchw_filter_layout", "return (((size_t)o * Cg + ci) * K + kh) * K + kw;", "return (((size_t)ci * O + o) * K + kh) * K + kw;", None),
    ("out_dim_ceil", "return span / s + 1;", "return (span + s - 1) / s + 1;", None),
]


def _replace_nth(text, old, new, nth):
    assert old in text, old
    if nth is None:
        return text.replace(old, new)
    pos = -1
    for _ in range(nth + 1):
        pos = text.index(old, pos + 1)
    return text[:pos] + new + text[pos + len(old):]


def _pin_calls():
    calls = []
    for case in TINY:
        calls.append(lambda c=case: test_fwd_equals_group_masked_dense_convolution(*c))
        calls.append(lambda c=case: test_bwd_data_equals_transposed_masked_dense_convolution(*c))
        calls.append(lambda c=case: test_bwd_filter_equals_masked_dense_gradient(*c))
    for case in TINY[:4]:
        calls.append(lambda c=case: test_nhwc_is_nchw_transposed(*c))
    calls.append(test_all_ones_closed_forms)
    calls.append(test_one_hot_filter_entry_pins_channel_and_shift)
    return calls


@pytest.mark.parametrize("name,old,new,nth", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, name, old, new, nth):
    src = open(SRC).read()
    mutated = _replace_nth(src, old, new, nth)
    assert mutated != src
    csrc = tmp_path / "mutant.c"
    csrc.write_text(mutated)
    lib_path = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-o", str(lib_path), str(csrc)])
    real = gconv._load()
    lib = ctypes.CDLL(str(lib_path))
    for fn in ("oracle_gconv_fwd", "oracle_gconv_bwd_data", "oracle_gconv_bwd_filter", "oracle_gconv_out_dims"):
        getattr(lib, fn).argtypes = getattr(real, fn).argtypes
        getattr(lib, fn).restype = getattr(real, fn).restype
    monkeypatch.setattr(gconv, "_lib", lib)
    caught = 0
    for call in _pin_calls():
        try:
            call()
        except (AssertionError, ValueError):
            caught += 1
    assert caught > 0, "no pin noticed the mutant %s" % name
