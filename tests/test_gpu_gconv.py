"""GPU parity of the group-convolution entry points (more than one channel per group), called through
the C ABI, against the CPU group oracle, element by element on seeded inputs."""
import numpy as np
import pytest
import torch

import paper_1803_09926_amd as dw
from oracle import gconv as og
from paper_1803_09926_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu

LAYOUTS = [wl.NCHW, wl.NHWC]
DTYPES = [wl.F32, wl.BF16]

# name, N, C, O, groups, H, W, K, stride, pad
CASES = [
    ("g2_small", 2, 8, 8, 4, 9, 11, 3, 1, 1),
    ("g4_k3s1", 3, 16, 16, 4, 20, 24, 3, 1, 1),
    ("g4_w56", 2, 8, 8, 2, 30, 56, 3, 1, 1),
    ("g8_k3s1", 2, 16, 16, 2, 14, 16, 3, 1, 1),
    ("g2_w112", 1, 4, 4, 2, 10, 112, 3, 1, 1),
    ("g4_tail14", 5, 32, 32, 8, 14, 14, 3, 1, 1),
    ("g4_tail7", 5, 32, 32, 8, 7, 7, 3, 1, 1),
    ("g4_28", 3, 24, 24, 6, 28, 28, 3, 1, 1),
    ("g4_odd_hw", 2, 8, 8, 2, 13, 15, 3, 1, 1),
    ("g4_w_not_mult4", 2, 8, 8, 2, 12, 18, 3, 1, 1),
    ("g3_odd_group", 2, 9, 9, 3, 10, 12, 3, 1, 1),
    ("cg4_og2", 2, 16, 8, 4, 12, 12, 3, 1, 1),
    ("cg2_og6", 2, 8, 24, 4, 12, 12, 3, 1, 1),
    ("g4_s2", 2, 16, 16, 4, 15, 16, 3, 2, 1),
    ("g4_s2_pad0", 2, 8, 8, 2, 12, 14, 3, 2, 0),
    ("g4_k5", 2, 8, 8, 2, 12, 12, 5, 1, 2),
    ("g2_k1", 2, 8, 8, 4, 6, 7, 1, 1, 0),
    ("one_group_dense", 2, 6, 10, 1, 9, 9, 3, 1, 1),
    ("g16", 1, 32, 32, 2, 12, 12, 3, 1, 1),
    ("depthwise_m1", 2, 16, 16, 16, 14, 14, 3, 1, 1),
    ("depthwise_m2", 2, 8, 16, 8, 12, 12, 3, 1, 1),
    ("g4_many_strips", 1, 8, 8, 2, 70, 28, 3, 1, 1),
    ("g4_wide", 1, 4, 4, 1, 5, 1100, 3, 1, 1),
    # channel counts per group that differ between the two sides, and tilings with ragged edges
    ("cg2_og4", 3, 8, 16, 4, 17, 20, 3, 1, 1),
    ("cg2_og8", 2, 4, 16, 2, 9, 12, 3, 1, 1),
    ("cg8_og2", 2, 16, 4, 2, 10, 14, 3, 1, 1),
    ("cg8_og8_w30", 3, 24, 24, 3, 33, 30, 3, 1, 1),
    ("cg4_c132_h40", 5, 132, 132, 33, 40, 6, 3, 1, 1),
    ("cg2_c6_tall", 7, 6, 6, 3, 61, 10, 3, 1, 1),
    ("cg4_h1", 2, 8, 8, 2, 1, 16, 3, 1, 1),
    ("cg4_w2", 2, 8, 8, 2, 9, 2, 3, 1, 1),
    # channel counts that are multiples of 64 with 4 or 8 channels per group: NHWC forward and backward-data run on
    # the matrix cores (last column quad partly outside the row, one strip and several, one row, one column)
    ("mm_cg4_c64_w14", 3, 64, 64, 16, 17, 14, 3, 1, 1),
    ("mm_cg4_c128_h40", 2, 128, 128, 32, 40, 9, 3, 1, 1),
    ("mm_cg8_c64_w13", 3, 64, 64, 8, 15, 13, 3, 1, 1),
    ("mm_cg8_c128_h33", 2, 128, 128, 16, 33, 6, 3, 1, 1),
    ("mm_cg4_h1", 2, 64, 64, 16, 1, 5, 3, 1, 1),
    # fewer channels than a wavefront's worth (several groups of four columns per wavefront), and groups of 2 (bf16)
    ("mm_cg4_c32_w37", 2, 32, 32, 8, 9, 37, 3, 1, 1),
    ("mm_cg8_c8_w70", 1, 8, 8, 1, 5, 70, 3, 1, 1),
    ("mm_cg2_c64_w30", 2, 64, 64, 32, 11, 30, 3, 1, 1),
    ("mm_cg2_c128", 1, 128, 128, 64, 7, 9, 3, 1, 1),
    ("mm_cg2_c16_w41", 3, 16, 16, 8, 6, 41, 3, 1, 1),
    ("mm_cg8_w1", 2, 64, 64, 8, 30, 1, 3, 1, 1),
    # NCHW rows of 7, 14 or 28 with 2, 4 or 8 channels per group: forward and backward-data stage whole groups in LDS
    # (last tile partly filled, planes that are not square, tiles of one group)
    ("sp_cg8_28", 3, 24, 24, 3, 28, 28, 3, 1, 1),
    ("sp_cg8_14_h9", 4, 16, 16, 2, 9, 14, 3, 1, 1),
    ("sp_cg2_14", 5, 12, 12, 6, 14, 14, 3, 1, 1),
    ("sp_cg4_h20_w28", 2, 20, 20, 5, 20, 28, 3, 1, 1),
    ("sp_cg8_7", 9, 16, 16, 2, 7, 7, 3, 1, 1),
    ("sp_cg8_h32_w7", 2, 8, 8, 1, 32, 7, 3, 1, 1),
    # NHWC stride 2 on the matrix cores (forward any size, backward-data on even maps): odd and even maps, a last column
    # quad partly outside the row, several strips, the smallest map
    ("mm_s2_cg4_c64_odd", 2, 64, 64, 16, 15, 16, 3, 2, 1),
    ("mm_s2_cg4_c128_even", 3, 128, 128, 32, 16, 12, 3, 2, 1),
    ("mm_s2_cg8_c128", 2, 128, 128, 16, 18, 10, 3, 2, 1),
    ("mm_s2_cg8_c64_odd", 2, 64, 64, 8, 9, 7, 3, 2, 1),
    ("mm_s2_tiny", 1, 64, 64, 16, 2, 2, 3, 2, 1),
    ("mm_s2_tall", 1, 128, 128, 32, 60, 4, 3, 2, 1),
    # NCHW stride 2 on small planes (even maps with rows of 14 or 28): all three passes stage whole groups in LDS
    ("sp_s2_cg4_28", 3, 24, 24, 6, 28, 28, 3, 2, 1),
    ("sp_s2_cg8_14", 4, 16, 16, 2, 14, 14, 3, 2, 1),
    ("sp_s2_cg2_h20_w14", 2, 12, 12, 6, 20, 14, 3, 2, 1),
    ("sp_s2_cg4_h6_w28", 5, 20, 20, 5, 6, 28, 3, 2, 1),
    ("sp_s2_cg8_h32_w28", 1, 8, 8, 1, 32, 28, 3, 2, 1),
]


def run_gpu(case, layout, dtype, x, w, dy):
    name, N, C, O, G, H, W, K, s, p = case
    d = dw.group_desc(N, C, H, W, K, s, p, G, O, layout, dtype)
    tdt = torch.float32 if dtype == wl.F32 else torch.bfloat16
    xt, wt, dyt = gu.to_dev(x, dtype), gu.to_dev(w, dtype), gu.to_dev(dy, dtype)
    y = torch.full(dy.shape, float("nan"), device="cuda", dtype=tdt)
    dx = torch.full(x.shape, float("nan"), device="cuda", dtype=tdt)
    dwt = torch.full(w.shape, float("nan"), device="cuda", dtype=torch.float32)
    wsb = torch.full((max(dw.gconv_bwd_filter_workspace_bytes(d), 16),), 0xFF, device="cuda", dtype=torch.uint8)
    dw.gconv_fwd(d, xt, wt, y)
    dw.gconv_bwd_data(d, dyt, wt, dx)
    dw.gconv_bwd_filter(d, xt, dyt, dwt, wsb)
    torch.cuda.synchronize()
    return y, dx, dwt


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
@pytest.mark.parametrize("layout", LAYOUTS, ids=["nchw", "nhwc"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_group_conv_matches_oracle(case, layout, dtype):
    name, N, C, O, G, H, W, K, s, p = case
    print("case", name, "layout", layout, "dtype", dtype, flush=True)
    x, w, dy = wl.make_group_inputs(N, C, O, G, H, W, K, s, p, layout, dtype, seed=1234)
    y, dx, dwt = run_gpu(case, layout, dtype, x, w, dy)
    kw = dict(K=K, stride=s, pad=p, groups=G, O=O, layout=layout, nthreads=8)
    tol = gu.TOL_F32 if dtype == wl.F32 else gu.TOL_BF16
    tag = "%s layout=%d dtype=%d" % (name, layout, dtype)
    gu.assert_close(gu.to_host(y), og.fwd(x, w, **kw), tol, "gconv fwd " + tag)
    gu.assert_close(gu.to_host(dx), og.bwd_data(dy, w, x_shape=x.shape, **kw), tol, "gconv bwd_data " + tag)
    gu.assert_close(gu.to_host(dwt), og.bwd_filter(x, dy, **kw), gu.TOL_F32_FILTER, "gconv bwd_filter " + tag)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
def test_group_nhwc_exchange_kernels_forced_tilings(dtype):
    """The lane-exchange NHWC kernels pick several images per block and whole-column strips only on large
    tensors; the tiling overrides force those paths (ragged last image group, ragged last strip, shallow and deep
    prefetch, two channels per lane) at sizes the oracle checks element by element."""
    cases = [("x_cg4", 5, 24, 24, 6, 13, 10, 3, 1, 1), ("x_cg8", 7, 16, 16, 2, 11, 9, 3, 1, 1)]
    knobs = [
        {"DWCONV_TUNE_GXNI": "3", "DWCONV_TUNE_GXTH": "5", "DWCONV_TUNE_GHWNI": "3", "DWCONV_TUNE_GHWTH": "5"},
        {"DWCONV_TUNE_GXNI": "2", "DWCONV_TUNE_GXPF": "2", "DWCONV_TUNE_GHWNI": "4"},
        {"DWCONV_TUNE_GXNI": "8", "DWCONV_TUNE_GXTH": "4", "DWCONV_TUNE_GHWTH": "3", "DWCONV_TUNE_GHWNI": "1"},
    ]
    for case in cases:
        name, N, C, O, G, H, W, K, s, p = case
        x, w, dy = wl.make_group_inputs(N, C, O, G, H, W, K, s, p, wl.NHWC, dtype, seed=99)
        kw = dict(K=K, stride=s, pad=p, groups=G, O=O, layout=wl.NHWC, nthreads=8)
        want = (og.fwd(x, w, **kw), og.bwd_data(dy, w, x_shape=x.shape, **kw), og.bwd_filter(x, dy, **kw))
        tol = gu.TOL_F32 if dtype == wl.F32 else gu.TOL_BF16
        for kn in knobs:
            if name == "x_cg8" and kn.get("DWCONV_TUNE_GXV") == "2":
                continue
            kn = dict(kn, DWCONV_TUNE_GMFMA="0")        # channel counts the matrix-core walk would take otherwise
            with dw.tuning_overrides(kn):
                print("case", name, "knobs", kn, flush=True)
                y, dx, dwt = run_gpu(case, wl.NHWC, dtype, x, w, dy)
            tag = "%s %s dtype=%d" % (name, kn, dtype)
            gu.assert_close(gu.to_host(y), want[0], tol, "gconv fwd " + tag)
            gu.assert_close(gu.to_host(dx), want[1], tol, "gconv bwd_data " + tag)
            gu.assert_close(gu.to_host(dwt), want[2], gu.TOL_F32_FILTER, "gconv bwd_filter " + tag)
    # two channels per lane (groups of 4 over two lanes)
    case = cases[0]
    name, N, C, O, G, H, W, K, s, p = case
    x, w, dy = wl.make_group_inputs(N, C, O, G, H, W, K, s, p, wl.NHWC, dtype, seed=98)
    kw = dict(K=K, stride=s, pad=p, groups=G, O=O, layout=wl.NHWC, nthreads=8)
    with dw.tuning_overrides({"DWCONV_TUNE_GXV": "2", "DWCONV_TUNE_GMFMA": "0"}):
        y, dx, dwt = run_gpu(case, wl.NHWC, dtype, x, w, dy)
    tol = gu.TOL_F32 if dtype == wl.F32 else gu.TOL_BF16
    gu.assert_close(gu.to_host(y), og.fwd(x, w, **kw), tol, "gconv fwd two channels per lane")
    gu.assert_close(gu.to_host(dx), og.bwd_data(dy, w, x_shape=x.shape, **kw), tol, "gconv bwd_data two channels per lane")


def test_group_nhwc_bf16_filter_gradient_dot_product_form_forced_tilings():
    """bf16 NHWC filter gradient with 2 or 4 channels per group: the row-pair dot-product kernels.  Strips of one, an odd
    and an even number of rows, ragged last strips and image groups, odd and even heights, a lane with 2 and with 4
    output channels."""
    cases = [("d2_cg2", 5, 12, 12, 6, 13, 10, 3, 1, 1), ("d2_cg2_og4", 3, 8, 16, 4, 8, 9, 3, 1, 1),
             ("d2_cg4", 4, 16, 16, 4, 7, 12, 3, 1, 1), ("d2_h1", 2, 8, 8, 4, 1, 5, 3, 1, 1), ("d2_h2", 2, 8, 8, 2, 2, 3, 3, 1, 1)]
    knobs = [{}, {"DWCONV_TUNE_GHWTH": "1"}, {"DWCONV_TUNE_GHWTH": "2", "DWCONV_TUNE_GHWNI": "2"},
             {"DWCONV_TUNE_GHWTH": "3", "DWCONV_TUNE_GHWNI": "3"}, {"DWCONV_TUNE_GHWTH": "4", "DWCONV_TUNE_GHWNI": "8"},
             {"DWCONV_TUNE_GHWTH": "64"}]
    for case in cases:
        name, N, C, O, G, H, W, K, s, p = case
        x, w, dy = wl.make_group_inputs(N, C, O, G, H, W, K, s, p, wl.NHWC, wl.BF16, seed=77)
        kw = dict(K=K, stride=s, pad=p, groups=G, O=O, layout=wl.NHWC, nthreads=8)
        want = og.bwd_filter(x, dy, **kw)
        for kn in knobs:
            with dw.tuning_overrides(kn):
                print("case", name, "knobs", kn, flush=True)
                _, _, dwt = run_gpu(case, wl.NHWC, wl.BF16, x, w, dy)
            gu.assert_close(gu.to_host(dwt), want, gu.TOL_F32_FILTER, "gconv bwd_filter %s %s" % (name, kn))
        with dw.tuning_overrides({"DWCONV_TUNE_GNODOT2": "1"}):
            _, _, dwt = run_gpu(case, wl.NHWC, wl.BF16, x, w, dy)
        gu.assert_close(gu.to_host(dwt), want, gu.TOL_F32_FILTER, "gconv bwd_filter multiply-add form " + name)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
def test_group_nchw_matrix_core_kernels_forced_tilings(dtype):
    """NCHW forward, backward-data and filter gradient of 14x14 (four images per fill, batches that are not multiples of
    four), 28x28 and 56x56 planes with 4 or 8 channels per group and of
    112x112 planes with 2 (matrix cores, planes or 14-row
    strips staged in LDS): blocks that take one image or strip, several, and a ragged share of them; one channel octet
    and several."""
    cases = [("mf_cg8", 5, 16, 16, 2, 28, 28, 3, 1, 1), ("mf_cg4", 7, 24, 24, 6, 28, 28, 3, 1, 1), ("mf_cg8_n1", 1, 8, 8, 1, 28, 28, 3, 1, 1),
             ("mf56_cg8", 2, 8, 8, 1, 56, 56, 3, 1, 1), ("mf56_cg4", 3, 16, 16, 4, 56, 56, 3, 1, 1),
             ("mf112_cg2", 2, 16, 16, 8, 112, 112, 3, 1, 1),
             ("mf14_cg8", 6, 16, 16, 2, 14, 14, 3, 1, 1), ("mf14_cg4", 9, 24, 24, 6, 14, 14, 3, 1, 1), ("mf14_n1", 1, 8, 8, 2, 14, 14, 3, 1, 1)]
    knobs = [{}, {"DWCONV_TUNE_GSMBLOCKS": "1", "DWCONV_TUNE_GSMFBLOCKS": "1"}, {"DWCONV_TUNE_GSMBLOCKS": "4", "DWCONV_TUNE_GSMFBLOCKS": "3"},
             {"DWCONV_TUNE_GSMBLOCKS": "9", "DWCONV_TUNE_GSMFBLOCKS": "7"}]
    tol = gu.TOL_F32 if dtype == wl.F32 else gu.TOL_BF16
    for case in cases:
        name, N, C, O, G, H, W, K, s, p = case
        x, w, dy = wl.make_group_inputs(N, C, O, G, H, W, K, s, p, wl.NCHW, dtype, seed=55)
        kw = dict(K=K, stride=s, pad=p, groups=G, O=O, layout=wl.NCHW, nthreads=8)
        want = (og.fwd(x, w, **kw), og.bwd_data(dy, w, x_shape=x.shape, **kw), og.bwd_filter(x, dy, **kw))
        d = dw.group_desc(N, C, H, W, K, s, p, G, O, wl.NCHW, dtype)
        assert dw.gconv_variant_name(d, 0) == "group_nchw_smallplane_mfma_k3s1"
        assert dw.gconv_variant_name(d, 1) == "group_nchw_smallplane_mfma_k3s1_flip"
        if W < 112 or dtype == wl.BF16:         # 112-wide fp32 filter gradient: the row walk, unless asked for
            assert dw.gconv_variant_name(d, 2) == "group_nchw_smallplane_mfma_bwd_filter_k3s1"
        for kn in knobs:
            kn = dict(kn, DWCONV_TUNE_GSMM112F32="1")
            with dw.tuning_overrides(kn):
                print("case", name, "knobs", kn, flush=True)
                assert dw.gconv_variant_name(d, 2) == "group_nchw_smallplane_mfma_bwd_filter_k3s1"
                y, dx, dwt = run_gpu(case, wl.NCHW, dtype, x, w, dy)
            tag = "%s %s" % (name, kn)
            gu.assert_close(gu.to_host(y), want[0], tol, "gconv fwd " + tag)
            gu.assert_close(gu.to_host(dx), want[1], tol, "gconv bwd_data " + tag)
            gu.assert_close(gu.to_host(dwt), want[2], gu.TOL_F32_FILTER, "gconv bwd_filter " + tag)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
def test_group_nhwc_lds_matrix_core_filter_gradient_forced_tilings(dtype):
    """NHWC filter gradient of 28x28 and 56x56 maps with 4 or 8 channels per group: the channels of an octet are scattered to
    planes in LDS and the sums run on the matrix cores.  Blocks with one fill, several and a ragged share; one octet and
    several; against the lane-exchange kernels as well."""
    cases = [("nl_cg8", 5, 16, 16, 2, 28, 28, 3, 1, 1), ("nl_cg4", 7, 24, 24, 6, 28, 28, 3, 1, 1), ("nl_cg8_n1", 1, 8, 8, 1, 28, 28, 3, 1, 1),
             ("nl56_cg8", 2, 8, 8, 1, 56, 56, 3, 1, 1), ("nl56_cg4", 3, 16, 16, 4, 56, 56, 3, 1, 1)]
    knobs = [{}, {"DWCONV_TUNE_GSMBLOCKS": "1"}, {"DWCONV_TUNE_GSMBLOCKS": "4"}, {"DWCONV_TUNE_GSMBLOCKS": "9"}]
    for case in cases:
        name, N, C, O, G, H, W, K, s, p = case
        x, w, dy = wl.make_group_inputs(N, C, O, G, H, W, K, s, p, wl.NHWC, dtype, seed=56)
        kw = dict(K=K, stride=s, pad=p, groups=G, O=O, layout=wl.NHWC, nthreads=8)
        want = og.bwd_filter(x, dy, **kw)
        d = dw.group_desc(N, C, H, W, K, s, p, G, O, wl.NHWC, dtype)
        # chosen by default for bf16 groups of 8 only; the switch asks for it everywhere
        assert (dw.gconv_variant_name(d, 2) == "group_nhwc_lds_mfma_bwd_filter_k3s1") == (dtype == wl.BF16 and C // G == 8)
        for kn in knobs:
            kn = dict(kn, DWCONV_TUNE_GSMMNHWCALL="1")
            with dw.tuning_overrides(kn):
                print("case", name, "knobs", kn, flush=True)
                assert dw.gconv_variant_name(d, 2) == "group_nhwc_lds_mfma_bwd_filter_k3s1"
                _, _, dwt = run_gpu(case, wl.NHWC, dtype, x, w, dy)
            gu.assert_close(gu.to_host(dwt), want, gu.TOL_F32_FILTER, "gconv bwd_filter %s %s" % (name, kn))
        with dw.tuning_overrides({"DWCONV_TUNE_GNOSMMNHWC": "1"}):
            assert dw.gconv_variant_name(d, 2) == "group_nhwc_bwd_filter_k3s1"
            _, _, dwt = run_gpu(case, wl.NHWC, dtype, x, w, dy)
        gu.assert_close(gu.to_host(dwt), want, gu.TOL_F32_FILTER, "gconv bwd_filter earlier kernels " + name)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
def test_group_nhwc_transposing_matrix_core_filter_gradient_forced_tilings(dtype):
    """NHWC filter gradient with 4 or 8 channels per group and whole wavefronts of channels: 4x4 tiles transposed in
    registers, sums on the matrix cores.  One image per wavefront and several, a ragged last image group, maps narrower
    than a block's 16 columns and wider, a single row, a single column."""
    cases = [("tr_cg4", 5, 128, 128, 32, 13, 21, 3, 1, 1), ("tr_cg8", 7, 128, 128, 16, 11, 7, 3, 1, 1), ("tr_cg8_c256", 3, 256, 256, 32, 6, 35, 3, 1, 1),
             ("tr_cg4_h1", 2, 128, 128, 32, 1, 9, 3, 1, 1), ("tr_cg8_w1", 2, 128, 128, 16, 9, 1, 3, 1, 1)]
    knobs = [{}, {"DWCONV_TUNE_GTRNI": "2"}, {"DWCONV_TUNE_GTRNI": "3", "DWCONV_TUNE_GTRBLOCKS": "7"}, {"DWCONV_TUNE_GTRBLOCKS": "100000"}]
    for case in cases:
        name, N, C, O, G, H, W, K, s, p = case
        x, w, dy = wl.make_group_inputs(N, C, O, G, H, W, K, s, p, wl.NHWC, dtype, seed=57)
        kw = dict(K=K, stride=s, pad=p, groups=G, O=O, layout=wl.NHWC, nthreads=8)
        want = og.bwd_filter(x, dy, **kw)
        d = dw.group_desc(N, C, H, W, K, s, p, G, O, wl.NHWC, dtype)
        for kn in knobs:
            kn = dict(kn, DWCONV_TUNE_GTRALL="1")
            with dw.tuning_overrides(kn):
                print("case", name, "knobs", kn, flush=True)
                assert dw.gconv_variant_name(d, 2) == "group_nhwc_mfma_bwd_filter_k3s1"
                _, _, dwt = run_gpu(case, wl.NHWC, dtype, x, w, dy)
            gu.assert_close(gu.to_host(dwt), want, gu.TOL_F32_FILTER, "gconv bwd_filter %s %s" % (name, kn))


def test_group_bwd_filter_is_deterministic():
    case = ("det", 4, 32, 32, 8, 28, 28, 3, 1, 1)
    for layout in LAYOUTS:
        x, w, dy = wl.make_group_inputs(*case[1:], layout, wl.F32, seed=7)
        a = run_gpu(case, layout, wl.F32, x, w, dy)[2]
        b = run_gpu(case, layout, wl.F32, x, w, dy)[2]
        assert torch.equal(a, b)


@pytest.mark.parametrize("ci", [6, 7], ids=["f32_b128", "bf16_b256"])
def test_group_benchmark_workload_full_size_sampled(ci):
    """The group-convolution benchmark workloads at their full size, in the launch configuration bench.py times;
    oracle on sampled images (fwd, bwd_data: images are independent) and on sampled groups over the whole batch
    (bwd_filter: groups are independent)."""
    cfg = wl.config(ci)
    N = cfg["N"]
    tol = gu.TOL_F32 if cfg["dtype"] == wl.F32 else gu.TOL_BF16
    for li, (layer, _) in enumerate(cfg["layers"]):
        for layout in cfg["layouts"]:
            print("group workload", layer.name, "layout", layout, flush=True)
            C, G, Cg = layer.C, layer.groups, layer.cg
            x, w, dy = wl.make_inputs_device(layer, N, layout, cfg["dtype"], seed=1000 * ci + li)
            d = dw.group_desc(N, C, layer.H, layer.W, 3, 1, 1, G, C, layout, cfg["dtype"])
            y = torch.full_like(dy, float("nan")); dx = torch.full_like(x, float("nan"))
            dwt = torch.full(w.shape, float("nan"), device="cuda", dtype=torch.float32)
            wsb = torch.full((max(dw.gconv_bwd_filter_workspace_bytes(d), 16),), 0xFF, device="cuda", dtype=torch.uint8)
            dw.gconv_fwd(d, x, w, y); dw.gconv_bwd_data(d, dy, w, dx); dw.gconv_bwd_filter(d, x, dy, dwt, wsb)
            torch.cuda.synchronize()
            tag = "%s layout=%d" % (layer.name, layout)
            kw = dict(K=3, stride=1, pad=1, groups=G, O=C, layout=layout, nthreads=8)
            wh = gu.to_host(w)
            imgs = sorted({0, N // 2 - 1, N - 1})
            xh, dyh = gu.to_host(x[imgs]), gu.to_host(dy[imgs])
            gu.assert_close(gu.to_host(y[imgs]), og.fwd(xh, wh, **kw), tol, "gconv fwd " + tag)
            gu.assert_close(gu.to_host(dx[imgs]), og.bwd_data(dyh, wh, x_shape=xh.shape, **kw), tol, "gconv bwd_data " + tag)
            kw1 = dict(K=3, stride=1, pad=1, groups=1, O=Cg, layout=layout, nthreads=8)
            for gi in sorted({0, G // 2 + 1 if G > 2 else 0, G - 1}):
                sl = slice(gi * Cg, (gi + 1) * Cg)
                if layout == wl.NCHW:
                    xc, dyc, got = gu.to_host(x[:, sl]), gu.to_host(dy[:, sl]), gu.to_host(dwt[sl])
                else:
                    xc, dyc, got = gu.to_host(x[..., sl]), gu.to_host(dy[..., sl]), gu.to_host(dwt[..., sl])
                gu.assert_close(got, og.bwd_filter(xc, dyc, **kw1), gu.TOL_F32_FILTER, "gconv bwd_filter group %d %s" % (gi, tag))
            del x, w, dy, y, dx, dwt
            torch.cuda.empty_cache()


def test_group_conv_writes_nothing_outside_its_outputs():
    G_ = 256
    for dtype in DTYPES:
        tdt = torch.float32 if dtype == wl.F32 else torch.bfloat16
        for layout in LAYOUTS:
            for case in [("gb1", 3, 8, 8, 2, 13, 12, 3, 1, 1), ("gb2", 2, 16, 16, 8, 9, 14, 3, 1, 1), ("gb3", 2, 12, 12, 4, 7, 9, 3, 2, 1)]:
                name, N, C, O, G, H, W, K, s, p = case
                x, w, dy = wl.make_group_inputs(N, C, O, G, H, W, K, s, p, layout, dtype, seed=3)
                xt, wt, dyt = gu.to_dev(x, dtype), gu.to_dev(w, dtype), gu.to_dev(dy, dtype)
                d = dw.group_desc(N, C, H, W, K, s, p, G, O, layout, dtype)

                def guarded(n, dt):
                    n_pad = (n + 7) // 8 * 8
                    buf = torch.full((n_pad + 2 * G_,), 12345.0, device="cuda", dtype=dt)
                    return buf, buf[G_:G_ + n]
                ybuf, yv = guarded(dy.size, tdt)
                dxbuf, dxv = guarded(x.size, tdt)
                dwbuf, dwv = guarded(w.size, torch.float32)
                wsb = torch.zeros(max(dw.gconv_bwd_filter_workspace_bytes(d), 16), device="cuda", dtype=torch.uint8)
                dw.gconv_fwd(d, xt, wt, yv); dw.gconv_bwd_data(d, dyt, wt, dxv); dw.gconv_bwd_filter(d, xt, dyt, dwv, wsb)
                torch.cuda.synchronize()
                for buf, v in [(ybuf, yv), (dxbuf, dxv), (dwbuf, dwv)]:
                    n = v.numel()
                    assert (buf[:G_] == 12345.0).all() and (buf[G_ + n:] == 12345.0).all(), (name, layout, dtype)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
def test_group_nhwc_matrix_core_kernels_forced_tilings(dtype):
    """The matrix-core NHWC kernels walk several images per wavefront only on large batches; the tiling overrides force
    that path (ragged last image group) and short strips (ragged last strip) at sizes the oracle checks element by
    element."""
    cases = [("mmx_cg4", 5, 128, 128, 32, 13, 10, 3, 1, 1), ("mmx_cg8", 7, 128, 128, 16, 11, 7, 3, 1, 1),
             ("mmx_cg2_c64", 5, 64, 64, 32, 13, 21, 3, 1, 1), ("mmx_cg4_c16", 7, 16, 16, 4, 11, 35, 3, 1, 1)]
    knobs = [{"DWCONV_TUNE_GMNI": "2", "DWCONV_TUNE_GMTH": "5"}, {"DWCONV_TUNE_GMNI": "3"}, {"DWCONV_TUNE_GMTH": "3"}]
    knobs = [dict(kn, DWCONV_TUNE_GMFMA2F32="1") for kn in knobs]       # groups of 2 in fp32 too (bf16 by default)
    for case in cases:
        name, N, C, O, G, H, W, K, s, p = case
        if C // G > 2 or dtype == wl.BF16:
            assert dw.gconv_variant_name(dw.group_desc(N, C, H, W, K, s, p, G, O, wl.NHWC, dtype), 0) == "group_nhwc_mfma_k3s1"
        x, w, dy = wl.make_group_inputs(N, C, O, G, H, W, K, s, p, wl.NHWC, dtype, seed=97)
        kw = dict(K=K, stride=s, pad=p, groups=G, O=O, layout=wl.NHWC, nthreads=8)
        want = (og.fwd(x, w, **kw), og.bwd_data(dy, w, x_shape=x.shape, **kw))
        tol = gu.TOL_F32 if dtype == wl.F32 else gu.TOL_BF16
        for kn in knobs:
            with dw.tuning_overrides(kn):
                print("case", name, "knobs", kn, flush=True)
                y, dx, _ = run_gpu(case, wl.NHWC, dtype, x, w, dy)
            tag = "%s %s dtype=%d" % (name, kn, dtype)
            gu.assert_close(gu.to_host(y), want[0], tol, "gconv fwd " + tag)
            gu.assert_close(gu.to_host(dx), want[1], tol, "gconv bwd_data " + tag)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
def test_group_nhwc_stride2_filter_gradient_forced_tilings(dtype):
    """The stride-2 NHWC filter gradient splits the dy rows into strips and walks several images per block only on large
    tensors; the tiling overrides force strips of 1, 3 and 4 rows (the row above a strip's first dy row comes from the
    neighbouring strip's range) and ragged image groups, on odd and even maps, against the oracle."""
    cases = [("s2w_cg4", 5, 24, 24, 6, 13, 10, 3, 2, 1), ("s2w_cg8", 3, 16, 16, 2, 12, 9, 3, 2, 1)]
    knobs = [{"DWCONV_TUNE_GHWTH": "1"}, {"DWCONV_TUNE_GHWTH": "3", "DWCONV_TUNE_GHWNI": "2"}, {"DWCONV_TUNE_GHWTH": "4", "DWCONV_TUNE_GHWNI": "8"}]
    for case in cases:
        name, N, C, O, G, H, W, K, s, p = case
        assert dw.gconv_variant_name(dw.group_desc(N, C, H, W, K, s, p, G, O, wl.NHWC, dtype), 2) == "group_nhwc_bwd_filter_k3s2"
        x, w, dy = wl.make_group_inputs(N, C, O, G, H, W, K, s, p, wl.NHWC, dtype, seed=96)
        kw = dict(K=K, stride=s, pad=p, groups=G, O=O, layout=wl.NHWC, nthreads=8)
        want = og.bwd_filter(x, dy, **kw)
        for kn in knobs:
            with dw.tuning_overrides(kn):
                print("case", name, "knobs", kn, flush=True)
                _, _, dwt = run_gpu(case, wl.NHWC, dtype, x, w, dy)
            gu.assert_close(gu.to_host(dwt), want, gu.TOL_F32_FILTER, "gconv bwd_filter %s %s dtype=%d" % (name, kn, dtype))
