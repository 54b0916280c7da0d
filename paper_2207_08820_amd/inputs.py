"""Seeded synthetic workloads (shapes and value ranges only; none of the method's arithmetic).

The paper evaluates trained ResNet-18 / YOLOv5 models on public datasets; neither the weights
nor the data are used here.  These generators take only the layer SHAPES and the VALUE RANGES
of those workloads: every tensor is uniform over the full range of its bit width, drawn from
``numpy.random.Generator(PCG64(seed))``.  The same arrays are handed to the CPU oracle and to
the GPU library by the tests and the benchmark.

Seed recipe: ``BASE + 10 * config + tensor_index`` (0 activations, 1 weights, 2 scale), plus
``1000 * layer`` for per-layer tensors of a stack.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_BASE = 220708 * 100

UNSIGNED, TWOS, BIPOLAR = 0, 1, 2


def seed_for(config: int, tensor_index: int, layer: int = 0) -> int:
    return SEED_BASE + 10 * config + tensor_index + 1000 * layer


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def value_bounds(bits: int, enc: int):
    if enc == UNSIGNED:
        return 0, (1 << bits) - 1
    if enc == TWOS:
        return -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    if enc == BIPOLAR:
        return -1, 1
    raise ValueError("unknown encoding")


def uniform_values(shape, bits: int, enc: int, seed: int) -> np.ndarray:
    """int8 array uniform over the encoding's full range (bipolar: uniform over {-1, +1})."""
    rng = _rng(seed)
    if enc == BIPOLAR:
        return (2 * rng.integers(0, 2, size=shape, dtype=np.int8) - 1).astype(np.int8)
    lo, hi = value_bounds(bits, enc)
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int8)


def uniform_scale(n: int, seed: int, lo: float = 0.01, hi: float = 0.1) -> np.ndarray:
    return _rng(seed).uniform(lo, hi, size=n).astype(np.float32)


@dataclass(frozen=True)
class GemmCase:
    M: int
    N: int
    K: int
    abits: int
    wbits: int
    enc_a: int
    enc_w: int


@dataclass(frozen=True)
class ConvLayer:
    """One conv of a stack.  ``src`` is the index of the layer whose requantized output is this
    layer's input (-1: the stack input)."""
    name: str
    H: int
    W: int
    Ci: int
    Co: int
    k: int
    stride: int
    pad: int
    src: int

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.k) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.k) // self.stride + 1

    @property
    def M(self) -> int:
        return self.Ho * self.Wo

    @property
    def K(self) -> int:
        return self.k * self.k * self.Ci

    @property
    def macs(self) -> int:
        return self.M * self.Co * self.K


# ---- config 1: one GEMM, the im2col of a 3x3x64 conv ------------------------------------------
CONFIG1 = GemmCase(64, 64, 576, 2, 2, UNSIGNED, UNSIGNED)


def config1():
    c = CONFIG1
    a = uniform_values((c.M, c.K), c.abits, c.enc_a, seed_for(1, 0))
    w = uniform_values((c.N, c.K), c.wbits, c.enc_w, seed_for(1, 1))
    return c, a, w


# ---- config 2: one ResNet-18-style 3x3 conv ----------------------------------------------------
CONFIG2 = ConvLayer("conv3x3_56x56x64", 56, 56, 64, 64, 3, 1, 1, -1)


def config2():
    L = CONFIG2
    x = uniform_values((1, L.H, L.W, L.Ci), 2, UNSIGNED, seed_for(2, 0))
    w = uniform_values((L.Co, L.k, L.k, L.Ci), 2, TWOS, seed_for(2, 1))
    scale = uniform_scale(L.Co, seed_for(2, 2))
    return L, x, w, scale


# ---- config 3: ResNet-18 basic-block conv stack at 224x224 (stem excluded) ---------------------
def resnet18_stack():
    """19 convs.  The sixteen 3x3 convs form one chain; each 1x1 stride-2 conv reads the same
    input as its stage's stride-2 3x3 conv and feeds nothing (no residual adds)."""
    layers = []
    side, ch = 56, 64
    prev = -1
    for stage, width in enumerate((64, 128, 256, 512)):
        for block in range(2):
            for conv in range(2):
                first = stage > 0 and block == 0 and conv == 0
                stride = 2 if first else 1
                layers.append(ConvLayer(f"s{stage}b{block}c{conv}_3x3", side, side, ch, width, 3, stride, 1, prev))
                idx = len(layers) - 1
                if first:
                    layers.append(ConvLayer(f"s{stage}_down_1x1", side, side, ch, width, 1, 2, 0, prev))
                    side //= 2
                    ch = width
                prev = idx
    return layers


# ---- config 4: YOLOv5s-style backbone shapes at 640x640 ----------------------------------------
def yolo_style_stack(bottlenecks: bool = False):
    """16 convs built from the widths 32/64/128/256/512 at strides 2..32 only: per stage one 3x3
    stride-2 conv C/2 -> C, then three 1x1 convs C -> C/2, C/2 -> C/2 and C -> C.  A synthetic
    stand-in for the shapes of such a backbone, not a copy of any model definition.
    bottlenecks: each stage also gets a 3x3 stride-1 conv C/2 -> C/2 on the inner 1x1 conv's output
    (20 convs)."""
    layers = []
    side, prev = 320, -1
    for C in (64, 128, 256, 512):
        layers.append(ConvLayer(f"c{C}_3x3s2", side, side, C // 2, C, 3, 2, 1, prev))
        down = len(layers) - 1
        side //= 2
        layers.append(ConvLayer(f"c{C}_split_1x1", side, side, C, C // 2, 1, 1, 0, down))
        layers.append(ConvLayer(f"c{C}_inner_1x1", side, side, C // 2, C // 2, 1, 1, 0, down + 1))
        if bottlenecks:
            layers.append(ConvLayer(f"c{C}_bneck_3x3", side, side, C // 2, C // 2, 3, 1, 1, down + 2))
        layers.append(ConvLayer(f"c{C}_merge_1x1", side, side, C, C, 1, 1, 0, down))
        prev = len(layers) - 1
    return layers


def stack_input(config: int, layers, batch: int = 1) -> np.ndarray:
    L = layers[0]
    return uniform_values((batch, L.H, L.W, L.Ci), 2, UNSIGNED, seed_for(config, 0))


def stack_weights(config: int, layers, wbits: int, enc_w: int):
    return [uniform_values((L.Co, L.k, L.k, L.Ci), wbits, enc_w, seed_for(config, 1, layer=i))
            for i, L in enumerate(layers)]


# ---- config 5: bit-width sweep of a large GEMM --------------------------------------------------
CONFIG5_PAIRS = ((1, 1), (2, 2), (3, 3), (4, 4), (2, 4))


def config5(abits: int, wbits: int, size: int = 4096):
    c = GemmCase(size, size, size, abits, wbits, UNSIGNED, TWOS)
    a = uniform_values((c.M, c.K), abits, UNSIGNED, seed_for(5, 0) + 100 * abits)
    w = uniform_values((c.N, c.K), wbits, TWOS, seed_for(5, 1) + 100 * wbits)
    return c, a, w
