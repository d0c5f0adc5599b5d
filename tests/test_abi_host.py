"""Host-side checks of the C ABI: the library loads, exports every symbol the header declares,
and every validation error is reported before any HIP call (so this runs with no GPU)."""
import ctypes
import os
import re

import pytest

import paper_1803_09926_amd as dw

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dwconv.h")

OK, E_NULL, E_DIM, E_ENUM, E_WS, E_ALIGN, E_UNSUP, E_LAUNCH, E_LARGE = 0, -1, -2, -3, -4, -5, -6, -7, -8
A, B, Cp, Dp = 0x1000, 0x2000, 0x3000, 0x4000   # fake aligned "device" addresses: never dereferenced on error paths


def test_library_exports_every_declared_symbol():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    declared = set(re.findall(r"\b((?:dwconv|gconv)_[a-z_]+)\s*\(", text))
    assert declared == set(dw.EXPORTS), declared ^ set(dw.EXPORTS)
    lib = dw.load()
    for name in declared:
        assert hasattr(lib, name), name


def test_desc_struct_matches_header_field_order():
    text = open(HEADER).read()
    body = re.search(r"typedef struct dwconv_desc \{(.*?)\} dwconv_desc;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in re.findall(r"int32_t\s+([^;]+);", body):
        fields += [f.strip() for f in decl.split(",")]
    assert fields == [f[0] for f in dw.Desc._fields_]
    assert ctypes.sizeof(dw.Desc) == 4 * len(fields)


def test_out_dims_follow_the_floor_formula():
    # MobileNet stride-2 chain of Table III: 112 -> 56 -> 28 -> 14 -> 7
    for H, Ho in [(112, 56), (56, 28), (28, 14), (14, 7)]:
        assert dw.out_dims(dw.desc(1, 8, H, H, 3, 2, 1)) == (Ho, Ho)
    assert dw.out_dims(dw.desc(1, 8, 7, 9, 3, 2, 1)) == (4, 5)
    assert dw.out_dims(dw.desc(1, 8, 2, 2, 3, 1, 1)) == (2, 2)       # map smaller than the filter, enough pad
    assert dw.out_dims(dw.desc(1, 8, 5, 5, 5, 1, 0)) == (1, 1)


@pytest.mark.parametrize("field,value,code", [
    ("N", 0, E_DIM), ("C", 0, E_DIM), ("H", -1, E_DIM), ("W", 0, E_DIM), ("K", 0, E_DIM), ("stride", 0, E_DIM),
    ("pad", -1, E_DIM), ("mult", 0, E_DIM), ("layout", 2, E_ENUM), ("layout", -1, E_ENUM), ("dtype", 2, E_ENUM),
    ("K", 16, E_UNSUP), ("N", 1 << 20, E_LARGE),
])
def test_bad_descriptors(field, value, code):
    d = dw.desc(2, 8, 16, 16)
    setattr(d, field, value)
    lib = dw.load()
    assert lib.dwconv_out_dims(ctypes.byref(d), None, None) == code
    assert lib.dwconv_fwd(ctypes.byref(d), A, B, Cp, None) == code
    assert lib.dwconv_bwd_data(ctypes.byref(d), A, B, Cp, None) == code
    assert lib.dwconv_bwd_filter(ctypes.byref(d), A, B, Cp, Dp, 1 << 30, None) == code
    assert lib.dwconv_bwd(ctypes.byref(d), A, B, Cp, Dp, 0x5000, 0x6000, 1 << 30, None) == code
    assert dw.bwd_filter_workspace_bytes(d) == 0
    assert dw.bwd_workspace_bytes(d) == 0
    assert dw.variant_name(d, 0) == "invalid"


def test_empty_output_is_a_bad_dim():
    d = dw.desc(1, 4, 2, 2, 5, 1, 0)     # 2 + 0 - 5 < 0
    assert dw.load().dwconv_out_dims(ctypes.byref(d), None, None) == E_DIM


def test_null_misaligned_and_workspace_errors():
    lib = dw.load()
    d = dw.desc(2, 8, 16, 16)
    ref = ctypes.byref(d)
    assert lib.dwconv_out_dims(None, None, None) == E_NULL
    assert lib.dwconv_fwd(None, A, B, Cp, None) == E_NULL
    for args in [(None, B, Cp), (A, None, Cp), (A, B, None)]:
        assert lib.dwconv_fwd(ref, *args, None) == E_NULL
        assert lib.dwconv_bwd_data(ref, *args, None) == E_NULL
        assert lib.dwconv_bwd_filter(ref, *args, Dp, 1 << 30, None) == E_NULL
    for args in [(A + 4, B, Cp), (A, B + 8, Cp), (A, B, Cp + 2)]:
        assert lib.dwconv_fwd(ref, *args, None) == E_ALIGN
        assert lib.dwconv_bwd_data(ref, *args, None) == E_ALIGN
        assert lib.dwconv_bwd_filter(ref, *args, Dp, 1 << 30, None) == E_ALIGN
    need = dw.bwd_filter_workspace_bytes(d)
    assert need > 0 and need <= (64 << 20)
    assert lib.dwconv_bwd_filter(ref, A, B, Cp, None, need, None) == E_WS
    assert lib.dwconv_bwd_filter(ref, A, B, Cp, Dp, need - 1, None) == E_WS
    assert lib.dwconv_bwd_filter(ref, A, B, Cp, Dp + 4, need, None) == E_ALIGN


def test_status_strings():
    seen = set()
    for code in range(0, -9, -1):
        s = dw.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 9
    assert dw.status_string(-99) == "unknown status"


def test_workspace_is_bounded_for_every_benchmark_layer():
    from paper_1803_09926_amd import workloads as wl
    for ci in range(5):
        cfg = wl.config(ci)
        for layer, _ in cfg["layers"]:
            for layout in cfg["layouts"]:
                d = dw.desc(cfg["N"], layer.C, layer.H, layer.W, layer.K, layer.stride, layer.pad, layer.mult,
                            layout, cfg["dtype"])
                assert dw.out_dims(d) == (layer.Ho, layer.Wo)
                need = dw.bwd_filter_workspace_bytes(d)
                assert 0 < need <= (64 << 20), (layer.name, need)
                for which in range(3):
                    assert dw.variant_name(d, which) not in ("", "invalid")


def test_benchmark_layers_get_tuned_variants():
    """No layer of the benchmark configurations (the five of the task and the MobileNet variant shapes) may
    fall back to the generic kernels, and none of the variant shapes to the slow LDS-tile kernels."""
    from paper_1803_09926_amd import workloads as wl
    for ci in range(6):
        cfg = wl.config(ci)
        for layer, _ in cfg["layers"]:
            for layout in cfg["layouts"]:
                d = dw.desc(cfg["N"], layer.C, layer.H, layer.W, layer.K, layer.stride, layer.pad, layer.mult,
                            layout, cfg["dtype"])
                for which in range(3):
                    name = dw.variant_name(d, which)
                    assert name != "generic", (ci, layer.name, layout, which)
                    if ci == 5:
                        assert not name.startswith("nchw_tile"), (ci, layer.name, layout, which, name)


def test_generic_fallback_is_selected_for_untuned_shapes():
    assert dw.variant_name(dw.desc(2, 6, 9, 9, 3, 1, 1, 1, dw.NHWC), 0) == "generic"       # C not a multiple of 4
    assert dw.variant_name(dw.desc(2, 8, 9, 9, 7, 1, 3, 1, dw.NCHW), 0) == "generic"       # 7x7
    assert dw.variant_name(dw.desc(2, 8, 9, 9, 3, 3, 1, 1, dw.NHWC), 2) == "generic"       # stride 3


def test_whole_backward_entry_point_validates_before_launch():
    lib = dw.load()
    for layout in (dw.NCHW, dw.NHWC):
        d = dw.desc(2, 8, 16, 16, 3, 1, 1, 1, layout)
        need = dw.bwd_workspace_bytes(d)
        assert 0 < need <= 64 << 20
        args = [A, B, Cp, Dp, 0x5000]
        for i in range(5):                                   # each of x, dy, w, dx, dw NULL in turn
            a = list(args); a[i] = None
            assert lib.dwconv_bwd(ctypes.byref(d), *a, 0x6000, need, None) == E_NULL
        assert lib.dwconv_bwd(ctypes.byref(d), A + 4, B, Cp, Dp, 0x5000, 0x6000, need, None) == E_ALIGN
        assert lib.dwconv_bwd(ctypes.byref(d), A, B, Cp, Dp, 0x5000, None, need, None) == E_WS
        assert lib.dwconv_bwd(ctypes.byref(d), A, B, Cp, Dp, 0x5000, 0x6000, need - 1, None) == E_WS


def test_whole_backward_variant_names():
    # fused kernels: NHWC 3x3 stride 1 and 2, NCHW 3x3 stride 1 (row-walk shapes, small planes) and fp32 stride 2 on row-walk
    # shapes; everything else runs the two passes
    assert dw.variant_name(dw.desc(128, 32, 112, 112, 3, 1, 1, 1, dw.NHWC, dw.F32), 3) == "nhwc_bwd_fused_k3s1"
    assert dw.variant_name(dw.desc(128, 64, 112, 112, 3, 2, 1, 1, dw.NHWC, dw.F32), 3) == "nhwc_bwd_fused_k3s2"
    assert dw.variant_name(dw.desc(4, 64, 115, 116, 3, 2, 1, 1, dw.NHWC, dw.F32), 3) == "separate"     # odd height
    assert dw.variant_name(dw.desc(128, 128, 56, 56, 3, 2, 1, 1, dw.NHWC, dw.F32), 3) == "nhwc_bwd_fused_k3s2"
    assert dw.variant_name(dw.desc(128, 32, 112, 112, 3, 1, 1, 1, dw.NCHW, dw.F32), 3) == "nchw_bwd_fused_k3s1"
    assert dw.variant_name(dw.desc(128, 512, 14, 14, 3, 1, 1, 1, dw.NCHW, dw.F32), 3) == "nchw_smallplane_bwd_fused_k3s1"
    assert dw.variant_name(dw.desc(128, 512, 14, 14, 3, 2, 1, 1, dw.NCHW, dw.F32), 3) == "nchw_smallplane_bwd_fused_k3s2"
    assert dw.variant_name(dw.desc(128, 256, 28, 28, 3, 2, 1, 1, dw.NCHW, dw.F32), 3) == "nchw_smallplane_bwd_fused_k3s2"
    assert dw.variant_name(dw.desc(256, 256, 28, 28, 3, 2, 1, 1, dw.NCHW, dw.BF16), 3) == "nchw_smallplane_bwd_fused_k3s2"
    assert dw.variant_name(dw.desc(8, 40, 7, 7, 3, 2, 1, 1, dw.NCHW, dw.F32), 3) == "separate"           # odd planes at stride 2
    # 28-wide rows at stride 1: fp32 rows are whole 16-byte vectors (row walk), bf16 rows take the small-plane kernel
    assert dw.variant_name(dw.desc(128, 256, 28, 28, 3, 1, 1, 1, dw.NCHW, dw.F32), 3) == "nchw_bwd_fused_k3s1"
    assert dw.variant_name(dw.desc(256, 256, 28, 28, 3, 1, 1, 1, dw.NCHW, dw.BF16), 3) == "nchw_smallplane_bwd_fused_k3s1"
    assert dw.variant_name(dw.desc(128, 64, 112, 112, 3, 2, 1, 1, dw.NCHW, dw.F32), 3) == "nchw_bwd_fused_k3s2"
    assert dw.variant_name(dw.desc(128, 64, 112, 112, 3, 2, 1, 1, dw.NCHW, dw.BF16), 3) == "nchw_bwd_fused_k3s2"
    assert dw.variant_name(dw.desc(128, 128, 56, 56, 3, 2, 1, 1, dw.NCHW, dw.BF16), 3) == "separate"      # bf16 rows under 112
    assert dw.variant_name(dw.desc(128, 32, 112, 112, 3, 1, 1, 1, dw.NCHW, dw.BF16), 3) == "nchw_bwd_fused_k3s1"
    assert dw.variant_name(dw.desc(128, 32, 112, 112, 5, 1, 2, 1, dw.NCHW, dw.BF16), 3) == "separate"                    # 5x5
    assert dw.variant_name(dw.desc(2, 6, 9, 9, 3, 1, 1, 1, dw.NHWC, dw.F32), 3) == "separate"
    # channel multiplier 2 (stride 1): the stride-1 kernel with two outputs per input channel
    assert dw.variant_name(dw.desc(32, 256, 56, 56, 3, 1, 1, 2, dw.NHWC, dw.F32), 3) == "nhwc_bwd_fused_k3s1_m2"
    assert dw.variant_name(dw.desc(32, 6, 12, 12, 3, 1, 1, 2, dw.NHWC, dw.BF16), 3) == "nhwc_bwd_fused_k3s1_m2"
    assert dw.variant_name(dw.desc(32, 256, 56, 56, 3, 2, 1, 2, dw.NHWC, dw.F32), 3) == "separate"
    assert dw.variant_name(dw.desc(32, 256, 56, 56, 3, 1, 1, 2, dw.NCHW, dw.F32), 3) == "separate"
    # bf16 NHWC: the fused kernels with four channels per lane
    assert dw.variant_name(dw.desc(256, 512, 14, 14, 3, 1, 1, 1, dw.NHWC, dw.BF16), 3) == "nhwc_bwd_fused_k3s1"
    assert dw.variant_name(dw.desc(256, 512, 14, 14, 3, 2, 1, 1, dw.NHWC, dw.BF16), 3) == "nhwc_bwd_fused_k3s2"
    assert dw.variant_name(dw.desc(256, 128, 56, 56, 3, 1, 1, 1, dw.NHWC, dw.BF16), 3) == "nhwc_bwd_fused_k3s1"
    assert dw.variant_name(dw.desc(256, 128, 56, 56, 5, 1, 2, 1, dw.NHWC, dw.BF16), 3) == "separate"


def test_buffer_view_kernels_stay_within_two_gib_images():
    # the bf16 5x5 NHWC kernels address an image through a 32-bit buffer view: an image above 2 GiB goes to the
    # generic kernels, an image of exactly 2 GiB and every 3x3 shape keep the row walk
    big = dw.desc(1, 8192, 512, 257, 5, 1, 2, 1, dw.NHWC, dw.BF16)
    assert [dw.variant_name(big, i) for i in range(3)] == ["generic"] * 3
    edge = dw.desc(1, 16384, 256, 256, 5, 1, 2, 1, dw.NHWC, dw.BF16)
    assert dw.variant_name(edge, 0) == "nhwc_rowwalk_k5s1" and dw.variant_name(edge, 1) == "nhwc_rowwalk_k5s1_flip"
    k3 = dw.desc(1, 16384, 256, 256, 3, 1, 1, 1, dw.NHWC, dw.F32)          # a 4 GiB image
    assert dw.variant_name(k3, 0) == "nhwc_rowwalk_k3s1" and dw.variant_name(k3, 2) == "nhwc_bwd_filter_k3s1"


# ---- group convolution entry points --------------------------------------------------------------------

def test_group_desc_struct_matches_header_field_order():
    text = open(HEADER).read()
    body = re.search(r"typedef struct dwconv_group_desc \{(.*?)\} dwconv_group_desc;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in re.findall(r"int32_t\s+([^;]+);", body):
        fields += [f.strip() for f in decl.split(",")]
    assert fields == [f[0] for f in dw.GroupDesc._fields_]
    assert ctypes.sizeof(dw.GroupDesc) == 4 * len(fields)


@pytest.mark.parametrize("field,value,code", [
    ("N", 0, E_DIM), ("C", 0, E_DIM), ("H", 0, E_DIM), ("W", -3, E_DIM), ("K", 0, E_DIM), ("stride", 0, E_DIM),
    ("pad", -1, E_DIM), ("groups", 0, E_DIM), ("O", 0, E_DIM), ("groups", 3, E_DIM), ("O", 10, E_DIM),
    ("layout", 2, E_ENUM), ("dtype", -1, E_ENUM), ("K", 16, E_UNSUP), ("N", 1 << 20, E_LARGE),
])
def test_group_bad_descriptors(field, value, code):
    d = dw.group_desc(2, 8, 16, 16, groups=4, O=8)
    setattr(d, field, value)
    lib = dw.load()
    assert lib.gconv_out_dims(ctypes.byref(d), None, None) == code
    assert lib.gconv_fwd(ctypes.byref(d), A, B, Cp, None) == code
    assert lib.gconv_bwd_data(ctypes.byref(d), A, B, Cp, None) == code
    assert lib.gconv_bwd_filter(ctypes.byref(d), A, B, Cp, Dp, 1 << 30, None) == code
    assert dw.gconv_bwd_filter_workspace_bytes(d) == 0
    assert dw.gconv_variant_name(d, 0) == "invalid"


def test_group_null_misaligned_and_workspace_errors():
    lib = dw.load()
    for layout in (dw.NCHW, dw.NHWC):
        for groups in (2, 8):                    # 4 channels per group, and the depthwise special case
            d = dw.group_desc(2, 8, 16, 16, groups=groups, O=8, layout=layout)
            ref = ctypes.byref(d)
            assert lib.gconv_fwd(None, A, B, Cp, None) == E_NULL
            for args in [(None, B, Cp), (A, None, Cp), (A, B, None)]:
                assert lib.gconv_fwd(ref, *args, None) == E_NULL
                assert lib.gconv_bwd_data(ref, *args, None) == E_NULL
                assert lib.gconv_bwd_filter(ref, *args, Dp, 1 << 30, None) == E_NULL
            for args in [(A + 4, B, Cp), (A, B + 8, Cp), (A, B, Cp + 2)]:
                assert lib.gconv_fwd(ref, *args, None) == E_ALIGN
                assert lib.gconv_bwd_data(ref, *args, None) == E_ALIGN
                assert lib.gconv_bwd_filter(ref, *args, Dp, 1 << 30, None) == E_ALIGN
            need = dw.gconv_bwd_filter_workspace_bytes(d)
            assert 0 < need <= (64 << 20)
            assert lib.gconv_bwd_filter(ref, A, B, Cp, None, need, None) == E_WS
            assert lib.gconv_bwd_filter(ref, A, B, Cp, Dp, need - 1, None) == E_WS


def test_group_variants_and_depthwise_delegation():
    assert dw.gconv_out_dims(dw.group_desc(1, 8, 7, 9, 3, 2, 1, groups=2, O=4)) == (4, 5)
    # one channel per group is the depthwise layer (here with multiplier 2) and reports its variant
    d = dw.group_desc(128, 32, 112, 112, groups=32, O=32, layout=dw.NHWC)
    assert dw.gconv_variant_name(d, 0) == dw.variant_name(dw.desc(128, 32, 112, 112, layout=dw.NHWC), 0)
    d = dw.group_desc(8, 16, 20, 20, groups=16, O=32, layout=dw.NCHW)
    assert dw.gconv_variant_name(d, 2) == dw.variant_name(dw.desc(8, 16, 20, 20, mult=2), 2)
    # untuned group shapes fall back to the generic group kernels
    assert dw.gconv_variant_name(dw.group_desc(2, 12, 9, 9, 5, 1, 2, groups=4, O=12), 0) == "group_generic"
    assert dw.gconv_variant_name(dw.group_desc(2, 12, 9, 9, 3, 2, 1, groups=4, O=12, layout=dw.NHWC), 1) == "group_generic"


def test_group_benchmark_layers_get_tuned_variants():
    from paper_1803_09926_amd import workloads as wl
    cfg = wl.config(6)
    for layer, _ in cfg["layers"]:
        for layout in cfg["layouts"]:
            d = dw.group_desc(cfg["N"], layer.C, layer.H, layer.W, layer.K, layer.stride, layer.pad, layer.groups,
                              layer.O, layout, cfg["dtype"])
            assert dw.gconv_out_dims(d) == (layer.Ho, layer.Wo)
            assert 0 < dw.gconv_bwd_filter_workspace_bytes(d) <= (64 << 20)
            for which in range(3):
                name = dw.gconv_variant_name(d, which)
                assert name.startswith("group_") and name != "group_generic", (layer.name, layout, which, name)


def test_group_nchw_matrix_core_filter_gradient_selection_and_workspace():
    """28x28 and 56x56 NCHW planes with 4 or 8 channels per group on both sides take the matrix-core filter gradient; its
    partial sums (one per block and, for groups of 4, per plane half) stay within the workspace the query reports."""
    for N in (1, 3, 128, 1000):
        for cg, C in ((4, 256), (8, 256), (8, 8), (4, 24), (2, 64), (2, 8)):
            for dt in (dw.F32, dw.BF16):
                for hw, fills in (((112, (16 if dt == dw.F32 else 8) * N),) if cg == 2 else ((14, (N + 3) // 4), (28, N), (56, 4 * N))):
                    if N * C * hw * hw >= 2 ** 31:
                        continue
                    d = dw.group_desc(N, C, hw, hw, 3, 1, 1, groups=C // cg, O=C, layout=dw.NCHW, dtype=dt)
                    if hw == 112 and dt == dw.F32:          # stays with the row walk
                        assert dw.gconv_variant_name(d, 2) == "group_nchw_bwd_filter_k3s1"
                        continue
                    assert dw.gconv_variant_name(d, 2) == "group_nchw_smallplane_mfma_bwd_filter_k3s1"
                    nbytes = dw.gconv_bwd_filter_workspace_bytes(d)
                    J = C * cg * 9 * 4
                    assert nbytes % J == 0
                    parts = nbytes // J
                    per_octet = parts // (1 if cg == 8 else 2)
                    assert 1 <= per_octet <= fills and per_octet * (C // 8) <= max(512 + C // 8, C // 8)
    # other shapes keep the earlier kernels
    assert dw.gconv_variant_name(dw.group_desc(4, 16, 28, 28, 3, 1, 1, groups=8, O=16), 2) != "group_nchw_smallplane_mfma_bwd_filter_k3s1"
    assert dw.gconv_variant_name(dw.group_desc(4, 12, 28, 28, 3, 1, 1, groups=3, O=12), 2) != "group_nchw_smallplane_mfma_bwd_filter_k3s1"
    assert dw.gconv_variant_name(dw.group_desc(4, 16, 14, 28, 3, 1, 1, groups=4, O=16), 2) != "group_nchw_smallplane_mfma_bwd_filter_k3s1"
    assert dw.gconv_variant_name(dw.group_desc(4, 16, 28, 28, 3, 1, 1, groups=4, O=32), 2) != "group_nchw_smallplane_mfma_bwd_filter_k3s1"


def test_dpp_operands_are_not_written_just_before_they_are_read(tmp_path):
    """The lane-exchange group kernels write their DPP multiply-adds as inline assembly, where the compiler does
    not insert the wait states the hardware needs between a vector-ALU write of a register and a DPP read of it
    (two instructions).  Check the generated ISA: no DPP source register is the destination of one of the two
    preceding vector-ALU instructions."""
    import re
    import shutil
    import subprocess
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    src = os.path.join(ROOT, "paper_1803_09926_amd", "csrc", "gconv_nhwc_xchg.hip")
    out = str(tmp_path / "xchg.s")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=fast", "-Xclang", "-target-feature",
                    "-Xclang", "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", out, src],
                   check=True, capture_output=True, timeout=600)
    # instruction lines only (inline-assembly lines are not indented like the compiler's own)
    lines = [l.strip() for l in open(out)]
    lines = [l for l in lines if re.match(r"[a-z]+_[a-z0-9_]+( |$)", l)]
    ndpp = 0
    for i, l in enumerate(lines):
        m = re.match(r"v_\w+_dpp (v\d+), (v\d+)", l)
        if not m:
            continue
        ndpp += 1
        for k in (1, 2):
            p = lines[i - k]
            if p.startswith("s_nop"):
                break
            w = re.match(r"v_\w+ (v\d+)", p)
            assert not (w and w.group(1) == m.group(2)), "DPP read of %s right after its write: %r then %r" % (m.group(2), p, l)
    assert ndpp > 1000      # the kernels do use the DPP form


def _ws_bound(d):
    O = d.C * d.mult
    return max(64 << 20, O * d.K * d.K * 4)


def test_planner_terminates_and_bounds_the_workspace_on_extreme_shapes():
    """Valid descriptors with very many channels, very wide rows or one-pixel planes: the host-side planning
    (variant, workspace size, both backward plans) must return, name a variant, and keep the workspace within
    max(64 MiB, the size of dw)."""
    shapes = [
        # N, C, H, W, K, s, p, m
        (2, 65536, 1, 147, 3, 1, 1, 1), (8, 1024, 1, 5000, 3, 1, 1, 2), (1, 2097152, 1, 1, 3, 1, 1, 1),
        (1, 4194304, 1, 1, 3, 1, 1, 1), (1, 70000, 16, 16, 3, 1, 1, 1), (1, 70000, 16, 16, 3, 2, 1, 1),
        (1, 131072, 16, 16, 5, 1, 2, 1), (4, 8, 1, 60000, 3, 1, 1, 1), (1, 4, 30000, 1, 3, 1, 1, 1),
        (1, 65540, 2, 8000, 3, 1, 1, 1), (3, 100000, 7, 7, 3, 1, 1, 1), (3, 100000, 14, 14, 3, 2, 1, 1),
        (1, 8, 20000, 8, 5, 1, 2, 1), (16, 32768, 8, 8, 3, 1, 1, 2), (1, 1 << 20, 4, 4, 15, 1, 7, 1),
    ]
    for N, C, H, W, K, s, p, m in shapes:
        for layout in (dw.NCHW, dw.NHWC):
            for dtype in (dw.F32, dw.BF16):
                d = dw.desc(N, C, H, W, K, s, p, m, layout, dtype)
                tag = (N, C, H, W, K, s, p, m, layout, dtype)
                for which in range(4):
                    assert dw.variant_name(d, which) not in ("", "invalid"), tag
                assert 0 < dw.bwd_filter_workspace_bytes(d) <= _ws_bound(d), tag
                assert 0 < dw.bwd_workspace_bytes(d) <= _ws_bound(d), tag
                # a workspace that is too small is refused before any launch
                assert dw.load().dwconv_bwd_filter(ctypes.byref(d), A, B, Cp, Dp, 8, None) == E_WS, tag


def test_planner_sweep_of_channels_and_widths():
    for C in (4, 60, 1000, 4096, 65535, 65536, 65537, 300000):
        for W in (1, 7, 14, 16, 56, 148, 1000, 5000):
            for H in (1, 16):
                if C * H * W >= 1 << 30:
                    continue
                for layout in (dw.NCHW, dw.NHWC):
                    d = dw.desc(2, C, H, W, 3, 1, 1, 1, layout, dw.F32)
                    assert dw.variant_name(d, 2) != "invalid"
                    assert 0 < dw.bwd_filter_workspace_bytes(d) <= _ws_bound(d), (C, H, W, layout)
                    assert 0 < dw.bwd_workspace_bytes(d) <= _ws_bound(d), (C, H, W, layout)


def test_group_workspace_bound_on_extreme_shapes():
    for (N, C, O, G, H, W, K) in [(1, 65536, 65536, 8192, 4, 4, 15), (2, 4096, 8192, 512, 1, 3000, 3),
                                  (1, 262144, 262144, 65536, 2, 2, 3), (4, 64, 64, 16, 1, 40000, 3)]:
        for layout in (dw.NCHW, dw.NHWC):
            d = dw.group_desc(N, C, H, W, K, 1, K // 2, G, O, layout, dw.F32)
            bound = max(64 << 20, O * (C // G) * K * K * 4)
            assert 0 < dw.gconv_bwd_filter_workspace_bytes(d) <= bound, (N, C, O, G, H, W, K, layout)
            assert dw.gconv_variant_name(d, 2) != "invalid"


def test_tuning_variables_are_a_snapshot_behind_a_master_switch(monkeypatch):
    """No call reads the environment: a DWCONV_TUNE_* variable set after the library's first use changes nothing
    until dwconv_tuning_reload, and nothing at all without the master switch DWCONV_TUNE=1."""
    d = dw.desc(128, 128, 56, 56, 3, 1, 1, 1, dw.NHWC, dw.F32)
    assert dw.tuning_reload() == 0
    base = dw.bwd_filter_workspace_bytes(d)
    monkeypatch.setenv("DWCONV_TUNE_NI", "1")
    monkeypatch.setenv("DWCONV_TUNE_THW", "7")
    assert dw.bwd_filter_workspace_bytes(d) == base            # not read on the call
    assert dw.tuning_reload() == 0                             # master switch off: still nothing
    assert dw.bwd_filter_workspace_bytes(d) == base
    monkeypatch.setenv("DWCONV_TUNE", "1")
    assert dw.bwd_filter_workspace_bytes(d) == base            # still the old snapshot
    assert dw.tuning_reload() == 2
    forced = dw.bwd_filter_workspace_bytes(d)
    assert forced > base                                       # one image and 7 rows per block: more partials
    monkeypatch.setenv("DWCONV_TUNE_NI", "-5")                 # nonsense values are clamped, never negative
    monkeypatch.setenv("DWCONV_TUNE_THW", "99999999999")
    assert dw.tuning_reload() == 2
    assert 0 < dw.bwd_filter_workspace_bytes(d) <= 64 << 20
    monkeypatch.delenv("DWCONV_TUNE")
    assert dw.tuning_reload() == 0
    assert dw.bwd_filter_workspace_bytes(d) == base
    with dw.tuning_overrides({"DWCONV_TUNE_NI": 1, "DWCONV_TUNE_THW": 7}):
        assert dw.bwd_filter_workspace_bytes(d) == forced
    assert dw.bwd_filter_workspace_bytes(d) == base
