"""Seeded synthetic inputs and layer-shape lists for the evaluated workloads.

This module holds no arithmetic of the method (no GEMM, no checksum, no
selector): only random operands in their storage formats and the (M, N, K)
shapes of the networks.  It is the one module that both the tests of the GPU
path and the CPU checker draw inputs from, so it imports neither.

Stand-ins: the paper evaluates torchvision CNNs with ImageNet weights and
Facebook's DLRM (Sec. 6.2, "Workloads").  Only the layer shapes matter for the
timing and for the checksum invariant, so weights and activations here are
seeded random values with the distributions named in each generator.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

F16, BF16, I8 = "f16", "bf16", "i8"


# --------------------------------------------------------------------------- #
# storage formats
# --------------------------------------------------------------------------- #
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float array -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    w = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (w >> 16) & 1
    w = (w + 0x7FFF + lsb) >> 16
    return w.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round real values to the storage type: float16 array, bf16 bits (uint16) or int8."""
    if dtype == F16:
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16)
    if dtype == BF16:
        return to_bf16_bits(x)
    if dtype == I8:
        return np.ascontiguousarray(x).astype(np.int8)
    raise ValueError(dtype)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def random_matrix(shape, dtype: str, dist: str, seed: int) -> np.ndarray:
    """dist: 'uniform_pm1' U[-1,1], 'uniform_01' U[0,1], 'normal' N(0,1),
    'weights' N(0,0.02), 'int8' uniform integers in [-128,127]."""
    rng = _rng(seed)
    if dist == "int8" or dtype == I8:
        return rng.integers(-128, 128, size=shape, dtype=np.int64).astype(np.int8)
    if dist == "uniform_pm1":
        x = rng.uniform(-1.0, 1.0, size=shape)
    elif dist == "uniform_01":
        x = rng.uniform(0.0, 1.0, size=shape)
    elif dist == "normal":
        x = rng.standard_normal(size=shape, dtype=np.float32)
    elif dist == "weights":
        x = 0.02 * rng.standard_normal(size=shape, dtype=np.float32)
    else:
        raise ValueError(dist)
    return to_storage(x, dtype)


def gemm_operands(M, N, K, dtype, seed, dist_a="uniform_pm1", dist_b="uniform_pm1"):
    """(A, B): A is M x K, B is K x N in the paper's orientation (Sec. 2.1)."""
    A = random_matrix((M, K), dtype, dist_a, 2 * seed + 1)
    B = random_matrix((K, N), dtype, dist_b, 2 * seed + 2)
    return A, B


# --------------------------------------------------------------------------- #
# layer shapes
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class Layer:
    name: str
    M: int
    N: int
    K: int
    # convolution geometry (None for fully-connected layers)
    conv: "Conv | None" = None


@dataclass(frozen=True)
class Conv:
    batch: int
    H: int
    W: int
    Cin: int
    Cout: int
    KH: int
    KW: int
    stride: int
    pad: int

    @property
    def OH(self):
        return (self.H + 2 * self.pad - self.KH) // self.stride + 1

    @property
    def OW(self):
        return (self.W + 2 * self.pad - self.KW) // self.stride + 1


def _conv_layer(name, batch, H, W, Cin, Cout, k, stride, pad) -> Layer:
    c = Conv(batch, H, W, Cin, Cout, k, k, stride, pad)
    return Layer(name, batch * c.OH * c.OW, Cout, k * k * Cin, c)


def dlrm_layers(batch: int, top=(512, 1024, 1024, 512, 256, 1)) -> List[Layer]:
    """DLRM MLPs as GEMMs with M = batch.  Bottom MLP 13-512-256-64 (Sec. 6.2); the top
    MLP widths default to this build's benchmark configuration 512-1024-1024-512-256-1
    (the paper's own top MLP is 512-256-1 after its input layer)."""
    bottom = (13, 512, 256, 64)
    layers = []
    for i in range(len(bottom) - 1):
        layers.append(Layer(f"bot{i}", batch, bottom[i + 1], bottom[i]))
    for i in range(len(top) - 1):
        layers.append(Layer(f"top{i}", batch, top[i + 1], top[i]))
    return layers


def resnet50_layers(batch: int, H: int = 224, W: int = 224, with_fc: bool = False) -> List[Layer]:
    """The 53 convolutions of ResNet-50 (bottleneck blocks [3,4,6,3], stride on the 3x3
    convolution) lowered to GEMM shapes, in network order (within a block: the three
    convolutions, then the 1x1 projection on the shortcut if the block has one);
    optionally followed by the 2048->1000 classifier."""
    layers = [_conv_layer("conv1", batch, H, W, 3, 64, 7, 2, 3)]
    h, w = layers[0].conv.OH, layers[0].conv.OW
    h, w = (h + 2 - 3) // 2 + 1, (w + 2 - 3) // 2 + 1  # 3x3 max-pool, stride 2, pad 1
    cin = 64
    for stage, (planes, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3)), start=1):
        for b in range(blocks):
            stride = 2 if (b == 0 and stage > 1) else 1
            p = f"layer{stage}.{b}"
            layers.append(_conv_layer(p + ".conv1", batch, h, w, cin, planes, 1, 1, 0))
            layers.append(_conv_layer(p + ".conv2", batch, h, w, planes, planes, 3, stride, 1))
            h2, w2 = layers[-1].conv.OH, layers[-1].conv.OW
            layers.append(_conv_layer(p + ".conv3", batch, h2, w2, planes, planes * 4, 1, 1, 0))
            if b == 0:
                layers.append(_conv_layer(p + ".downsample", batch, h, w, cin, planes * 4, 1, stride, 0))
            h, w, cin = h2, w2, planes * 4
    if with_fc:
        layers.append(Layer("fc", batch, 1000, 2048))
    return layers


def square_sizes_paper():
    """M = N = K of the paper's square-GEMM study (Sec. 6.4, Fig. 11)."""
    return [32, 64, 128, 256, 512, 1024, 2048]


def sweep_m():
    """M values of the intensity sweep with N = K = 4096."""
    return [1 << i for i in range(14)]


def conv_operands(c: Conv, dtype: str, seed: int):
    """(x, Wmat): NHWC activations U[0,1] and the weight matrix K x N with k = (kh, kw, c),
    N(0, 0.02) (int8: uniform integers)."""
    x = random_matrix((c.batch, c.H, c.W, c.Cin), dtype, "uniform_01", 2 * seed + 1)
    Wm = random_matrix((c.KH * c.KW * c.Cin, c.Cout), dtype, "weights", 2 * seed + 2)
    return x, Wm
