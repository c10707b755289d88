"""Seeded synthetic convolution workloads.

This module only *describes* layers and draws their tensors; it contains none of
the convolution / Winograd arithmetic.  It is the one piece shared by the CPU
oracle's tests and the HIP path's tests and benchmark, so that both sides see
bit-identical inputs.

The five workload families stand in for the networks the paper evaluates
(MobileNet-v1, ResNet-18 and friends at one 224x224 image, Section 4.1): they
take the *layer shapes* of those networks and fill them with seeded random
tensors.  No dataset item, trained weight or model file is involved.

Recipe (all workloads):
  * generator   numpy ``Generator(PCG64(seed))``, seed = 200212418 + 1000*config + layer
  * draw order  x, then w, then b  (float64 draws, rounded once to float32)
  * x           uniform[lo, hi]   (``x_range`` of the workload)
  * w           normal(0, sqrt(2 / (kh*kw*C_in)))      (He-normal)
  * b           uniform[-0.1, 0.1]
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

BASE_SEED = 200212418


@dataclass(frozen=True)
class ConvLayer:
    """One 2-D convolution layer: NCHW input, KCRS weight, groups = 1."""
    name: str
    n: int
    c_in: int
    h: int
    w: int
    c_out: int
    kh: int
    kw: int
    stride: int = 1
    pad: object = 0              # int, or (pad_h, pad_w)
    dil: int = 1
    x_range: Tuple[float, float] = (-1.0, 1.0)
    seed: int = BASE_SEED

    @property
    def pad_hw(self) -> Tuple[int, int]:
        return tuple(self.pad) if isinstance(self.pad, (tuple, list)) else (self.pad, self.pad)

    @property
    def h_out(self) -> int:
        return (self.h + 2 * self.pad_hw[0] - self.dil * (self.kh - 1) - 1) // self.stride + 1

    @property
    def w_out(self) -> int:
        return (self.w + 2 * self.pad_hw[1] - self.dil * (self.kw - 1) - 1) // self.stride + 1

    @property
    def k_long(self) -> int:
        """Taps along the longer side of the kernel (the k of F(n, k) for square and single-row/column kernels)."""
        return max(self.kh, self.kw)

    @property
    def out_shape(self) -> Tuple[int, int, int, int]:
        return (self.n, self.c_out, self.h_out, self.w_out)

    @property
    def direct_flops(self) -> int:
        """2*N*K*C*H_o*W_o*kh*kw: the direct-convolution count every scheme is priced in."""
        return 2 * self.n * self.c_out * self.c_in * self.h_out * self.w_out * self.kh * self.kw

    def with_batch(self, n: int) -> "ConvLayer":
        return ConvLayer(self.name, n, self.c_in, self.h, self.w, self.c_out, self.kh, self.kw,
                         self.stride, self.pad, self.dil, self.x_range, self.seed)


def draw(layer: ConvLayer, with_bias: bool = True):
    """Return (x, w, b) as float32 numpy arrays for ``layer`` (b is None without bias)."""
    rng = np.random.Generator(np.random.PCG64(layer.seed))
    lo, hi = layer.x_range
    x = rng.uniform(lo, hi, size=(layer.n, layer.c_in, layer.h, layer.w)).astype(np.float32)
    sigma = float(np.sqrt(2.0 / (layer.kh * layer.kw * layer.c_in)))
    w = rng.normal(0.0, sigma, size=(layer.c_out, layer.c_in, layer.kh, layer.kw)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, size=(layer.c_out,)).astype(np.float32)
    return x, w, (b if with_bias else None)


def _mk(cfg: int, idx: int, name: str, n, c, hw, k, ksz, stride, pad, x_range=(-1.0, 1.0)) -> ConvLayer:
    return ConvLayer(name=name, n=n, c_in=c, h=hw, w=hw, c_out=k, kh=ksz, kw=ksz, stride=stride,
                     pad=pad, dil=1, x_range=x_range, seed=BASE_SEED + 1000 * cfg + idx)


def config_layers(cfg: int) -> List[ConvLayer]:
    """The layers of workload family ``cfg`` (1..5)."""
    if cfg == 1:
        return [_mk(1, 0, "c16_32x32_k3", 1, 16, 32, 16, 3, 1, 1)]
    if cfg in (2, 3):
        n = 1 if cfg == 2 else 32
        out = [
            _mk(cfg, 0, "res64_56x56_k3", n, 64, 56, 64, 3, 1, 1),
            _mk(cfg, 1, "res128_28x28_k3", n, 128, 28, 128, 3, 1, 1),
            _mk(cfg, 2, "res256_14x14_k3", n, 256, 14, 256, 3, 1, 1),
            _mk(cfg, 3, "res512_7x7_k3", n, 512, 7, 512, 3, 1, 1),
        ]
        if cfg == 2:
            out += [
                _mk(cfg, 4, "res64to128_56x56_k3s2", n, 64, 56, 128, 3, 2, 1),
                _mk(cfg, 5, "res128to256_28x28_k3s2", n, 128, 28, 256, 3, 2, 1),
                _mk(cfg, 6, "res256to512_14x14_k3s2", n, 256, 14, 512, 3, 2, 1),
            ]
        return out
    if cfg == 4:
        shapes = [(32, 64, 112), (64, 128, 56), (128, 256, 28), (256, 512, 14), (512, 1024, 7), (1024, 1024, 7)]
        return [_mk(4, i, f"pw{c}to{k}_{hw}x{hw}", 16, c, hw, k, 1, 1, 0, (0.0, 1.0))
                for i, (c, k, hw) in enumerate(shapes)]
    if cfg == 5:
        return [
            _mk(5, 0, "mix256_128x128_k3", 16, 256, 128, 256, 3, 1, 1),
            _mk(5, 1, "mix128_64x64_k5", 16, 128, 64, 128, 5, 1, 2),
            _mk(5, 2, "mix64_112x112_k7", 16, 64, 112, 64, 7, 1, 3),
        ]
    raise ValueError(f"unknown workload config {cfg}")


def chain_layers(kind: str, n: int = 1) -> List[ConvLayer]:
    """Layers that feed one another (layer i+1 takes layer i's output), for the chained execution path.

    ``resnet18_trunk``: the seven 3x3 layers of workload families 2/3 in network order -- a stride-1 layer at
    each of the four resolutions with the stride-2 transition between them -- at batch ``n``.
    ``small``: five small ragged layers (3x3, stride-2 3x3, 1x1, 5x5, unpadded 3x3) the oracle finishes quickly.
    Only each layer's w and b are drawn (``draw``); x is drawn for the first layer alone.
    """
    if kind == "resnet18_trunk":
        by_name = {l.name: l for l in config_layers(2)}
        order = ["res64_56x56_k3", "res64to128_56x56_k3s2", "res128_28x28_k3", "res128to256_28x28_k3s2",
                 "res256_14x14_k3", "res256to512_14x14_k3s2", "res512_7x7_k3"]
        return [by_name[nm].with_batch(n) for nm in order]
    if kind == "small":
        def L(i, name, c, h, w, k, ksz, s, p):
            return ConvLayer(name, n, c, h, w, k, ksz, ksz, s, p, 1, (-1.0, 1.0), BASE_SEED + 9500 + i)
        return [
            L(0, "ch0_k3", 5, 21, 18, 12, 3, 1, 1),        # -> 12 x 21 x 18
            L(1, "ch1_k3s2", 12, 21, 18, 9, 3, 2, 1),      # -> 9 x 11 x 9
            L(2, "ch2_pw", 9, 11, 9, 20, 1, 1, 0),         # -> 20 x 11 x 9
            L(3, "ch3_k5", 20, 11, 9, 6, 5, 1, 2),         # -> 6 x 11 x 9
            L(4, "ch4_k3nopad", 6, 11, 9, 7, 3, 1, 0),     # -> 7 x 9 x 7
        ]
    raise ValueError(f"unknown chain {kind!r}")


CONFIG_TITLES: Dict[int, str] = {
    1: "cfg1: single 3x3 conv 16->16 32x32 N=1",
    2: "cfg2: ResNet-18-style 3x3 layers N=1 (+stride-2 transitions)",
    3: "cfg3: ResNet-18-style 3x3 stride-1 layers N=32",
    4: "cfg4: MobileNet-v1-style pointwise 1x1 layers N=16",
    5: "cfg5: mixed-kernel stress 3x3/5x5/7x7 N=16",
}


def small_parity_layers() -> List[ConvLayer]:
    """Small ragged / edge layers the oracle finishes in well under a second each."""
    def L(i, name, n, c, h, w, k, kh, kw, s=1, p=0, d=1):
        return ConvLayer(name, n, c, h, w, k, kh, kw, s, p, d, (-1.0, 1.0), BASE_SEED + 9000 + i)
    return [
        L(0, "tiny_3x3", 1, 3, 6, 6, 2, 3, 3, 1, 1),
        L(1, "ragged_7x7_k3", 2, 5, 7, 7, 6, 3, 3, 1, 1),
        L(2, "ragged_14x9_k3", 3, 17, 14, 9, 33, 3, 3, 1, 1),
        L(3, "nopad_13x13_k3", 2, 8, 13, 13, 8, 3, 3, 1, 0),
        L(4, "k5_same_11x15", 2, 9, 11, 15, 7, 5, 5, 1, 2),
        L(5, "k7_same_16x16", 1, 4, 16, 16, 5, 7, 7, 1, 3),
        L(6, "k2_nopad_9x9", 2, 6, 9, 9, 4, 2, 2, 1, 0),
        L(7, "stride2_k3", 2, 12, 15, 15, 10, 3, 3, 2, 1),
        L(8, "dil2_k3", 1, 7, 12, 12, 9, 3, 3, 1, 2, 2),
        L(9, "pw_1x1_odd", 3, 19, 7, 7, 21, 1, 1, 1, 0),
        L(10, "pw_1x1_wide", 2, 40, 12, 12, 70, 1, 1, 1, 0),
        L(11, "multi_tile_k3", 2, 70, 30, 34, 130, 3, 3, 1, 1),
        L(12, "rect_1x7", 1, 5, 9, 20, 6, 1, 7, 1, 0),
        L(13, "pad_bigger_than_needed", 1, 4, 8, 8, 4, 3, 3, 1, 2),
        L(14, "rect_7x1_same", 2, 6, 17, 13, 9, 7, 1, 1, (3, 0)),
        L(15, "rect_1x3_same", 2, 10, 9, 22, 5, 1, 3, 1, (0, 1)),
        L(16, "rect_5x1_nopad", 1, 3, 23, 6, 4, 5, 1, 1, 0),
        L(17, "rect_3x5_same", 1, 4, 10, 12, 3, 3, 5, 1, (1, 2)),
        L(18, "rect_5x2_nopad", 2, 7, 14, 9, 6, 5, 2, 1, 0),
        L(19, "rect_2x7_pad", 1, 5, 11, 19, 9, 2, 7, 1, (1, 2)),
        L(20, "rect_4x3_ragged", 2, 9, 13, 15, 10, 4, 3, 1, (2, 1)),
    ]


def rect_layers(n: int = 16) -> List[ConvLayer]:
    """Factorised 7-tap layers (1x7 then 7x1, 'same' padding) on a 17x17 map, the shape of the
    Inception-style blocks the paper's benchmark networks contain; seeded like the workload families."""
    def L(i, name, c, k, kh, kw, pad):
        return ConvLayer(name, n, c, 17, 17, k, kh, kw, 1, pad, 1, (-1.0, 1.0), BASE_SEED + 9700 + i)
    return [
        L(0, "incep128_17x17_1x7", 128, 128, 1, 7, (0, 3)),
        L(1, "incep128_17x17_7x1", 128, 128, 7, 1, (3, 0)),
        L(2, "incep192_17x17_1x7", 192, 192, 1, 7, (0, 3)),
        L(3, "incep192_17x17_7x1", 192, 192, 7, 1, (3, 0)),
    ]


def selection_table_layers(n: int = 1) -> List[ConvLayer]:
    """The three convolution settings (k, i_c, o_c, size) of the paper's scheme-selection comparison (Table 1):
    (2, 3, 16, 224), (2, 512, 512, 16), (3, 64, 64, 112).  The paper states neither padding nor batch: no padding
    for the 2-tap kernels, 'same' padding for the 3-tap one, batch `n`."""
    def L(i, name, c, k, hw, kk, pad):
        return ConvLayer(name, n, c, hw, hw, k, kk, kk, 1, pad, 1, (-1.0, 1.0), BASE_SEED + 9800 + i)
    return [
        L(0, "sel3to16_224x224_k2", 3, 16, 224, 2, 0),
        L(1, "sel512_16x16_k2", 512, 512, 16, 2, 0),
        L(2, "sel64_112x112_k3", 64, 64, 112, 3, 1),
    ]
