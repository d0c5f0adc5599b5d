"""Seeded synthetic workloads: layer tables and input generators.

This module holds none of the method's arithmetic.  It names the layer shapes
(the thirteen depthwise layers of MobileNet-v1 as listed in the paper's Table III,
and Xception-style stride-1 layers), and draws x, w and dy from a seeded
generator.  Both the GPU tests and the CPU oracle consume the arrays it returns.

Recipe: x, dy ~ N(0,1); w ~ N(0, variance 1/K^2) (sigma = 1/K, so outputs have
about unit variance); float32; drawn in NCHW logical order and permuted for NHWC
so both layouts see the same values; for the bf16 workloads every array is then
rounded to the nearest bf16 (ties to even) and kept as float32 holding exactly
that value.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np

NCHW = 0
NHWC = 1
F32 = 0
BF16 = 1


@dataclass(frozen=True)
class Layer:
    name: str
    C: int
    H: int
    W: int
    K: int = 3
    stride: int = 1
    pad: int = 1
    mult: int = 1
    cg: int = 1          # input (= output) channels per group; 1 is the depthwise layer, > 1 a group convolution

    @property
    def O(self) -> int:
        return self.C * self.mult

    @property
    def groups(self) -> int:
        return self.C // self.cg

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.K) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.K) // self.stride + 1

    def x_elems(self, N: int) -> int:
        return N * self.C * self.H * self.W

    def y_elems(self, N: int) -> int:
        return N * self.O * self.Ho * self.Wo

    def pass_bytes(self, N: int, elem_bytes: int) -> int:
        """Algorithmic bytes one pass must move: every input element and every output element once."""
        return (self.x_elems(N) + self.y_elems(N)) * elem_bytes

    def pass_flops(self, N: int) -> int:
        return 2 * self.K * self.K * self.cg * self.y_elems(N)


def _mb(i, C, H, s):
    return Layer("mobilenet_dw%02d_c%d_h%d_s%d" % (i, C, H, s), C, H, H, 3, s, 1, 1)


# The thirteen depthwise layers of MobileNet-v1 (224 input, width 1.0): Table III's shapes.
MOBILENET_V1: Tuple[Layer, ...] = (
    _mb(1, 32, 112, 1), _mb(2, 64, 112, 2), _mb(3, 128, 56, 1), _mb(4, 128, 56, 2),
    _mb(5, 256, 28, 1), _mb(6, 256, 28, 2),
    _mb(7, 512, 14, 1), _mb(8, 512, 14, 1), _mb(9, 512, 14, 1), _mb(10, 512, 14, 1), _mb(11, 512, 14, 1),
    _mb(12, 512, 14, 2), _mb(13, 1024, 7, 1),
)


def _xc(name, C, H, mult=1):
    return Layer("xception_%s_c%d_h%d_m%d" % (name, C, H, mult), C, H, H, 3, 1, 1, mult)


# Xception-style stride-1 layers; `repeat` says how often the layer occurs in the stack.
XCEPTION: Tuple[Tuple[Layer, int], ...] = (
    (_xc("entry1", 128, 147), 1), (_xc("entry2", 256, 74), 1), (_xc("entry3", 728, 37), 1),
    (_xc("middle", 728, 19), 24),
    (_xc("exit1", 1024, 19), 1), (_xc("exit2", 1536, 10), 1), (_xc("exit3", 2048, 10), 1),
    (_xc("mult2", 256, 56, 2), 1),
)


def _gc(C, H, cg):
    return Layer("group_c%d_h%d_cg%d" % (C, H, cg), C, H, H, 3, 1, 1, 1, cg)


# Group convolutions (3x3, stride 1, as many output as input channels) on MobileNet-sized planes:
# 2, 4 and 8 channels per group.
GROUP_LAYERS: Tuple[Layer, ...] = (
    _gc(64, 112, 2), _gc(128, 56, 4), _gc(256, 28, 4), _gc(256, 28, 8), _gc(512, 14, 4),
)


def mobilenet_5x5() -> Tuple[Layer, ...]:
    """The nine stride-1 MobileNet layers with a 5x5 pad-2 filter."""
    return tuple(replace(l, name=l.name + "_k5", K=5, pad=2) for l in MOBILENET_V1 if l.stride == 1)


def mobilenet_variant(width: float = 1.0, resolution: int = 224, shallow: bool = False) -> Tuple[Layer, ...]:
    """Depthwise layers of the MobileNet variants of the paper's Table V: channels scaled by `width`
    (0.75 -> 24, 48, 96, ...; 0.5 -> 16, 32, ...), input resolution 224 or 128 (first depthwise layer
    at resolution/2), `shallow` drops the five 14x14x512 layers.  Shapes only."""
    out = []
    for i, l in enumerate(MOBILENET_V1, 1):
        if shallow and 7 <= i <= 11:
            continue
        C = int(round(l.C * width))
        H = l.H * resolution // 224
        out.append(Layer("mobilenet_w%g_r%d_dw%02d_c%d_h%d_s%d" % (width, resolution, i, C, H, l.stride),
                         C, H, H, 3, l.stride, 1, 1))
    return tuple(out)


def config(index: int) -> Dict:
    """The benchmark configurations, as dicts: N, layouts, dtype, layers [(Layer, repeat)].
    0..4: the five configurations of the benchmark spec; 5: the MobileNet variant shapes (width 0.75, width 0.5 at
    resolution 128), as a second workload; 6: group convolutions with 2, 4 and 8 channels per group on
    MobileNet-sized planes; 7: the same in bf16 storage at batch 256."""
    if index == 0:
        return dict(name="single_3x3_n8_c32_h112_f32_nchw", N=8, layouts=(NCHW,), dtype=F32,
                    layers=[(Layer("single_c32_h112", 32, 112, 112), 1)])
    if index == 1:
        return dict(name="mobilenet_v1_dw_b64_f32_nhwc", N=64, layouts=(NHWC,), dtype=F32,
                    layers=[(l, 1) for l in MOBILENET_V1])
    if index == 2:
        return dict(name="mobilenet_v1_dw_b128_f32_nchw_nhwc", N=128, layouts=(NCHW, NHWC), dtype=F32,
                    layers=[(l, 1) for l in MOBILENET_V1])
    if index == 3:
        return dict(name="xception_dw_b32_f32_nhwc", N=32, layouts=(NHWC,), dtype=F32,
                    layers=list(XCEPTION))
    if index == 4:
        return dict(name="mobilenet_v1_dw_b256_bf16", N=256, layouts=(NHWC, NCHW), dtype=BF16,
                    layers=[(l, 1) for l in MOBILENET_V1] + [(l, 1) for l in mobilenet_5x5()])
    if index == 5:
        return dict(name="mobilenet_variants_b128_f32", N=128, layouts=(NCHW, NHWC), dtype=F32,
                    layers=[(l, 1) for l in mobilenet_variant(0.75, 224)] +
                           [(l, 1) for l in mobilenet_variant(0.5, 128)])
    if index == 6:
        return dict(name="group_conv_b128_f32", N=128, layouts=(NCHW, NHWC), dtype=F32,
                    layers=[(l, 1) for l in GROUP_LAYERS])
    if index == 7:
        return dict(name="group_conv_b256_bf16", N=256, layouts=(NCHW, NHWC), dtype=BF16,
                    layers=[(l, 1) for l in GROUP_LAYERS])
    raise ValueError("config index must be 0..7")


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result is float32 holding that value."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """The upper 16 bits of float32 values that already hold exact bf16 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def make_inputs(layer: Layer, N: int, layout: int, dtype: int, seed: int):
    """Return (x, w, dy) as float32 numpy arrays in `layout`.

    x  [N,C,H,W] / [N,H,W,C];  dy [N,O,Ho,Wo] / [N,Ho,Wo,O];  w [O,K,K] / [K,K,O].
    """
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, layer.C, layer.H, layer.W), dtype=np.float32)
    w = rng.standard_normal((layer.O, layer.K, layer.K), dtype=np.float32) / np.float32(layer.K)
    dy = rng.standard_normal((N, layer.O, layer.Ho, layer.Wo), dtype=np.float32)
    if dtype == BF16:
        x, w, dy = round_to_bf16(x), round_to_bf16(w), round_to_bf16(dy)
    if layout == NHWC:
        x = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
        dy = np.ascontiguousarray(dy.transpose(0, 2, 3, 1))
        w = np.ascontiguousarray(w.transpose(1, 2, 0))
    return x, w, dy


def to_layout(a_nchw: np.ndarray, layout: int) -> np.ndarray:
    return a_nchw if layout == NCHW else np.ascontiguousarray(a_nchw.transpose(0, 2, 3, 1))


def w_to_layout(w_okk: np.ndarray, layout: int) -> np.ndarray:
    return w_okk if layout == NCHW else np.ascontiguousarray(w_okk.transpose(1, 2, 0))


def make_inputs_device(layer: Layer, N: int, layout: int, dtype: int, seed: int, device="cuda"):
    """Same recipe as make_inputs, drawn on the device with torch's seeded generator (for the
    full-size workloads, where host generation and the PCIe copy would dominate).  Returns torch
    tensors x, w, dy in `layout`, float32 or bfloat16 storage.  The values differ from
    make_inputs' (another generator); tests that use this copy what they sample back to the host."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    tdt = torch.float32 if dtype == F32 else torch.bfloat16
    if layout == NCHW:
        xs, ys, ws = (N, layer.C, layer.H, layer.W), (N, layer.O, layer.Ho, layer.Wo), (layer.O, layer.K, layer.K)
        if layer.cg > 1: ws = (layer.O, layer.cg, layer.K, layer.K)
    else:
        xs, ys, ws = (N, layer.H, layer.W, layer.C), (N, layer.Ho, layer.Wo, layer.O), (layer.K, layer.K, layer.O)
        if layer.cg > 1: ws = (layer.K, layer.K, layer.cg, layer.O)
    x = torch.randn(xs, generator=gen, device=device, dtype=torch.float32).to(tdt)
    w = (torch.randn(ws, generator=gen, device=device, dtype=torch.float32) / (layer.K * layer.cg ** 0.5)).to(tdt)
    dy = torch.randn(ys, generator=gen, device=device, dtype=torch.float32).to(tdt)
    return x, w, dy


def make_group_inputs(N, C, O, groups, H, W, K, stride, pad, layout, dtype, seed):
    """Inputs of a group convolution, as float32 numpy arrays in `layout`:
    x [N,C,H,W] / [N,H,W,C] ~ N(0,1);  w [O,Cg,K,K] / [K,K,Cg,O] ~ N(0, 1/(K*K*Cg));  dy ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    Cg = C // groups
    Ho = (H + 2 * pad - K) // stride + 1
    Wo = (W + 2 * pad - K) // stride + 1
    x = rng.standard_normal((N, C, H, W), dtype=np.float32)
    w = rng.standard_normal((O, Cg, K, K), dtype=np.float32) / np.float32(K * np.sqrt(Cg))
    dy = rng.standard_normal((N, O, Ho, Wo), dtype=np.float32)
    if dtype == BF16:
        x, w, dy = round_to_bf16(x), round_to_bf16(w), round_to_bf16(dy)
    if layout == NHWC:
        x = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
        dy = np.ascontiguousarray(dy.transpose(0, 2, 3, 1))
        w = np.ascontiguousarray(w.transpose(2, 3, 1, 0))
    return x, w, dy
