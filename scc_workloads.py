"""Seeded synthetic inputs for the SCC layer shapes that are measured and tested.

This module holds layer shapes and random draws only: none of the method's
arithmetic (no window index maths, no convolution).  It is the one module that
both the CPU oracle's tests and the GPU path's tests/benchmark import, so that
the two sides see identical arrays.

The shapes stand in for image-classification layers (CIFAR-10 / ImageNet sized
feature maps, Section 5.1 of the paper); the datasets themselves are not used.
Draws: numpy PCG64 (``default_rng``), float64 normal draws cast to float32.
Seed = 745000 + 100*config + 10*layer + {0: x, 1: w, 2: dy, 3: depthwise filters, 4: the block's input}.
"""
import math
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Layer:
    name: str
    config: int           # index used in the seed
    N: int
    Cin: int
    Cout: int
    H: int
    W: int
    cg: int
    co: float
    x_law: str = "normal"      # "normal" -> N(0,1); "halfnormal" -> |N(0,1)| (post-ReLU)
    w_std: float = 0.0         # 0 -> He: sqrt(2 / (Cin // cg))
    layer: int = 0

    @property
    def L(self):
        return self.Cin // self.cg

    @property
    def HW(self):
        return self.H * self.W


def seed_of(layer, which):
    return 745000 + 100 * layer.config + 10 * layer.layer + {"x": 0, "w": 1, "dy": 2, "kdw": 3, "xin": 4}[which]


def make_inputs(layer, seed_offset=0):
    """(x, w, dy) as float32 C-contiguous arrays for one layer."""
    def draw(which, shape):
        rng = np.random.default_rng(seed_of(layer, which) + 1000003 * seed_offset)
        return rng.standard_normal(shape)

    x = draw("x", (layer.N, layer.Cin, layer.H, layer.W))
    if layer.x_law == "halfnormal":
        x = np.abs(x)
    std = layer.w_std if layer.w_std > 0 else math.sqrt(2.0 / layer.L)
    w = draw("w", (layer.Cout, layer.L)) * std
    dy = draw("dy", (layer.N, layer.Cout, layer.H, layer.W))
    return (np.ascontiguousarray(x, dtype=np.float32),
            np.ascontiguousarray(w, dtype=np.float32),
            np.ascontiguousarray(dy, dtype=np.float32))


def make_block_inputs(layer, dw_stride=1, seed_offset=0):
    """(xin, kdw, w) for a DW + SCC block whose SCC stage is `layer`: the block's input map is the one a depthwise
    3x3 stage of spatial stride `dw_stride` turns into the layer's H x W map (H*stride x W*stride pixels),
    depthwise filters ~ N(0, 1/3) (nine taps: unit output variance), w as in make_inputs."""
    def draw(which, shape):
        rng = np.random.default_rng(seed_of(layer, which) + 1000003 * seed_offset)
        return rng.standard_normal(shape)

    xin = draw("xin", (layer.N, layer.Cin, layer.H * dw_stride, layer.W * dw_stride))
    if layer.x_law == "halfnormal":
        xin = np.abs(xin)
    kdw = draw("kdw", (layer.Cin, 3, 3)) / 3.0
    std = layer.w_std if layer.w_std > 0 else math.sqrt(2.0 / layer.L)
    w = draw("w", (layer.Cout, layer.L)) * std
    return (np.ascontiguousarray(xin, dtype=np.float32), np.ascontiguousarray(kdw, dtype=np.float32),
            np.ascontiguousarray(w, dtype=np.float32))


# configs[0]: the small case the oracle finishes instantly.
SMALL = Layer("c1_small", 1, N=1, Cin=32, Cout=32, H=8, W=8, cg=2, co=0.5, w_std=0.1)

# configs[1]: the layer the headline metric is quoted on, and its overlap sweep.
METRIC = Layer("c2_n128_c256_16x16_cg4_co50", 2, N=128, Cin=256, Cout=256, H=16, W=16, cg=4, co=0.5)
METRIC_SWEEP = [replace(METRIC, name="c2_n128_c256_16x16_cg4_co%02d" % round(100 * co), co=co)
                for co in (0.0, 0.25, 0.5, 0.75)]

# configs[2]: late-stage 14x14 layer, post-ReLU activations (fp32 and bf16).
LATE = Layer("c3_n64_c512_14x14_cg8_co50", 3, N=64, Cin=512, Cout=512, H=14, W=14, cg=8, co=0.5,
             x_law="halfnormal")

# configs[3]: channel-expanding layer whose windows wrap many times.
EXPAND = Layer("c4_n128_c128to512_32x32_cg2_co33", 4, N=128, Cin=128, Cout=512, H=32, W=32, cg=2, co=0.33)

# configs[4]: MobileNet-shaped stack (channels and spatial size after each
# block's depthwise stage).  The configuration text spells out twelve channel
# transitions and says thirteen blocks; the thirteenth is read as the final
# 1024 -> 1024 block of the MobileNet shape.
_STACK_SHAPES = [(32, 64, 32), (64, 128, 16), (128, 128, 16), (128, 256, 8), (256, 256, 8),
                 (256, 512, 4), (512, 512, 4), (512, 512, 4), (512, 512, 4), (512, 512, 4),
                 (512, 512, 4), (512, 1024, 2), (1024, 1024, 2)]
STACK = [Layer("c5_l%02d_%dto%d_%dx%d" % (i, ci, co_, s, s), 5, N=128, Cin=ci, Cout=co_, H=s, W=s,
               cg=2, co=0.5, layer=i) for i, (ci, co_, s) in enumerate(_STACK_SHAPES)]

ALL_FULL = METRIC_SWEEP + [LATE, EXPAND] + STACK
# spatial stride of the depthwise stage in front of each stack layer: 2 where the map halves (MobileNet shape)
STACK_DW_STRIDE = [1 if i == 0 or _STACK_SHAPES[i][2] == _STACK_SHAPES[i - 1][2] else 2 for i in range(len(_STACK_SHAPES))]

# The paper's other sweeps on the metric layer (Section 5.3): the number of channel groups cg in
# {1, 2, 4, 8} at 50% overlap, and the batch size from inference-sized 16 up to 1024.
# Seeds: config 6 (layer index = position in the cg sweep) and config 7 (position in the batch sweep).
CG_SWEEP = [replace(METRIC, name="c6_n128_c256_16x16_cg%d_co50" % cg, config=6, cg=cg, layer=i)
            for i, cg in enumerate((1, 2, 4, 8))]
BATCH_SWEEP = [replace(METRIC, name="c7_n%d_c256_16x16_cg4_co50" % n, config=7, N=n, layer=i)
               for i, n in enumerate((16, 32, 64, 128, 256, 512, 1024))]


def algorithmic_bytes(layer, elem_bytes=4):
    """Bytes one pass must move when every tensor crosses HBM exactly once."""
    return elem_bytes * (layer.N * layer.HW * (layer.Cin + layer.Cout) + layer.Cout * layer.L)


def algorithmic_flops(layer):
    """2 * MACs of one pass: only the banded work, never the dense Cin*Cout product."""
    return 2 * layer.N * layer.Cout * layer.L * layer.HW


def block_algorithmic_bytes(layer, dw_stride=1, elem_bytes=4):
    """Bytes the forward of a DW + SCC block must move: its input, its output and both sets of weights, once."""
    return elem_bytes * (layer.N * layer.Cin * layer.HW * dw_stride * dw_stride + layer.N * layer.Cout * layer.HW +
                         layer.Cout * layer.L + 9 * layer.Cin)
