"""Seeded synthetic inputs and workload shape tables.

This module is the only thing the CPU oracle's tests and the HIP path's tests /
benchmark have in common.  It holds no arithmetic of the method itself (no GEMM,
no convolution, no epilogue, no padding): it only draws tensors from a counter
based generator and lists problem shapes.  Neither the oracle nor the HIP
library imports the other; both are handed the FP16 bytes produced here.

Generator: splitmix64 applied to (seed-derived key + element counter); the top
24 bits give u in [0,1).  Uniform and normal draws are rounded once to FP16
(numpy's IEEE round-to-nearest-even conversion).

Workloads stand in for the paper's (ResNet-50 layer *shapes*, Table 1 / Table 2
shapes); no dataset item or trained weight is used anywhere.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 output function on an array of uint64 states (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def _unit(seed: int, tensor_id: int, n: int, stream: int = 0) -> np.ndarray:
    """n draws of u in [0,1) as float64, a pure function of (seed, tensor_id, stream, index)."""
    with np.errstate(over="ignore"):
        key = _splitmix64(np.array([(seed * 0x1000003 + tensor_id * 0x10001 + stream) & 0xFFFFFFFFFFFFFFFF],
                                   dtype=np.uint64))[0]
        ctr = np.arange(n, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15) + key
    bits = _splitmix64(ctr)
    return (bits >> np.uint64(40)).astype(np.float64) * (1.0 / (1 << 24))


def uniform_fp16(seed: int, tensor_id: int, shape, lo: float, hi: float) -> np.ndarray:
    n = int(np.prod(shape)) if len(shape) else 1
    u = _unit(seed, tensor_id, n)
    return (lo + (hi - lo) * u).astype(np.float32).astype(np.float16).reshape(shape)


def normal_fp16(seed: int, tensor_id: int, shape, std: float) -> np.ndarray:
    """Box-Muller on two independent streams, scaled by std, rounded to FP16."""
    n = int(np.prod(shape)) if len(shape) else 1
    u1 = _unit(seed, tensor_id, n, stream=1)
    u2 = _unit(seed, tensor_id, n, stream=2)
    u1 = np.maximum(u1, 1.0 / (1 << 25))
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (z * std).astype(np.float16).reshape(shape)


def integer_fp16(seed: int, tensor_id: int, shape, lo: int, hi: int) -> np.ndarray:
    """Integers in [lo, hi] (inclusive) stored as FP16: every product and partial sum stays exact."""
    n = int(np.prod(shape)) if len(shape) else 1
    u = _unit(seed, tensor_id, n)
    v = np.floor(lo + (hi - lo + 1) * u)
    return np.clip(v, lo, hi).astype(np.float16).reshape(shape)


# ----------------------------------------------------------------------------------------------
# Problem descriptions
# ----------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class GemmShape:
    M: int
    N: int
    K: int

    @property
    def flops(self) -> int:
        return 2 * self.M * self.N * self.K

    @property
    def bytes(self) -> int:
        return 2 * (self.M * self.K + self.K * self.N + self.M * self.N + self.N)


@dataclass(frozen=True)
class ConvShape:
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    c_logical: int = 0  # channels before padding to a multiple of 8 (0 = same as C)

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def gemm_m(self) -> int:
        return self.N * self.P * self.Q

    @property
    def gemm_k(self) -> int:
        return self.R * self.S * self.C

    @property
    def flops(self) -> int:
        """Useful FLOPs: counts the logical (unpadded) input channels."""
        c = self.c_logical or self.C
        return 2 * self.gemm_m * self.K * self.R * self.S * c

    @property
    def bytes(self) -> int:
        """Each tensor once, FP16; a strided 1x1 only counts the pixels it samples."""
        if self.R == 1 and self.S == 1 and self.pad == 0:
            x_elems = self.gemm_m * self.C
        else:
            x_elems = self.N * self.H * self.W * self.C
        return 2 * (x_elems + self.K * self.gemm_k + self.gemm_m * self.K + self.K)


def resnet50_layers(batch: int = 32) -> List[Tuple[ConvShape, int]]:
    """The 23 distinct conv shapes of a ResNet-50 (stride on the 3x3 of a down-sampling block)
    with their multiplicity among the 53 conv layers.  Stem channels 3 are padded to 8."""
    L: List[Tuple[ConvShape, int]] = []
    b = batch
    L.append((ConvShape(b, 224, 224, 8, 64, 7, 7, 2, 3, c_logical=3), 1))
    # stage 1 (56x56), in 64, mid 64, out 256, 3 blocks
    L.append((ConvShape(b, 56, 56, 64, 64, 1, 1, 1, 0), 1))
    L.append((ConvShape(b, 56, 56, 64, 64, 3, 3, 1, 1), 3))
    L.append((ConvShape(b, 56, 56, 64, 256, 1, 1, 1, 0), 4))     # 3 expand + 1 projection
    L.append((ConvShape(b, 56, 56, 256, 64, 1, 1, 1, 0), 2))
    # stage 2 (56 -> 28), mid 128, out 512, 4 blocks
    L.append((ConvShape(b, 56, 56, 256, 128, 1, 1, 1, 0), 1))
    L.append((ConvShape(b, 56, 56, 128, 128, 3, 3, 2, 1), 1))
    L.append((ConvShape(b, 28, 28, 128, 512, 1, 1, 1, 0), 4))
    L.append((ConvShape(b, 56, 56, 256, 512, 1, 1, 2, 0), 1))    # projection
    L.append((ConvShape(b, 28, 28, 512, 128, 1, 1, 1, 0), 3))
    L.append((ConvShape(b, 28, 28, 128, 128, 3, 3, 1, 1), 3))
    # stage 3 (28 -> 14), mid 256, out 1024, 6 blocks
    L.append((ConvShape(b, 28, 28, 512, 256, 1, 1, 1, 0), 1))
    L.append((ConvShape(b, 28, 28, 256, 256, 3, 3, 2, 1), 1))
    L.append((ConvShape(b, 14, 14, 256, 1024, 1, 1, 1, 0), 6))
    L.append((ConvShape(b, 28, 28, 512, 1024, 1, 1, 2, 0), 1))   # projection
    L.append((ConvShape(b, 14, 14, 1024, 256, 1, 1, 1, 0), 5))
    L.append((ConvShape(b, 14, 14, 256, 256, 3, 3, 1, 1), 5))
    # stage 4 (14 -> 7), mid 512, out 2048, 3 blocks
    L.append((ConvShape(b, 14, 14, 1024, 512, 1, 1, 1, 0), 1))
    L.append((ConvShape(b, 14, 14, 512, 512, 3, 3, 2, 1), 1))
    L.append((ConvShape(b, 7, 7, 512, 2048, 1, 1, 1, 0), 3))
    L.append((ConvShape(b, 14, 14, 1024, 2048, 1, 1, 2, 0), 1))  # projection
    L.append((ConvShape(b, 7, 7, 2048, 512, 1, 1, 1, 0), 2))
    L.append((ConvShape(b, 7, 7, 512, 512, 3, 3, 1, 1), 2))
    assert sum(c for _, c in L) == 53 and len(L) == 23
    return L


# ----------------------------------------------------------------------------------------------
# The five benchmark configurations: tensors as numpy FP16 arrays
# ----------------------------------------------------------------------------------------------
def config1(seed: int = 1) -> Dict[str, np.ndarray]:
    """GEMM + bias + ReLU, A[256x256], B[256x256] row-major, bias[256], U[-1,1]."""
    return dict(A=uniform_fp16(seed, 0, (256, 256), -1, 1),
                B=uniform_fp16(seed, 1, (256, 256), -1, 1),
                bias=uniform_fp16(seed, 2, (256,), -1, 1))


def conv_tensors(shape: ConvShape, seed: int, weight: str = "uniform") -> Dict[str, np.ndarray]:
    """x NHWC U[-1,1]; w KRSC either U[-1,1] or N(0, 2/fan_in) (variance); bias U[-1,1].
    Tensors carry the logical (unpadded) channel count; padding to a multiple of 8 is the job of
    the code under test."""
    c_log = shape.c_logical or shape.C
    x = uniform_fp16(seed, 0, (shape.N, shape.H, shape.W, c_log), -1, 1)
    if weight == "uniform":
        w = uniform_fp16(seed, 1, (shape.K, shape.R, shape.S, c_log), -1, 1)
    else:
        fan_in = shape.R * shape.S * c_log
        w = normal_fp16(seed, 1, (shape.K, shape.R, shape.S, c_log), float(np.sqrt(2.0 / fan_in)))
    bias = uniform_fp16(seed, 2, (shape.K,), -1, 1)
    return dict(x=x, w=w, bias=bias)


CONFIG2_SHAPE = ConvShape(32, 56, 56, 64, 64, 3, 3, 1, 1)


def config2(seed: int = 2, batch: int = 32) -> Dict[str, np.ndarray]:
    s = ConvShape(batch, 56, 56, 64, 64, 3, 3, 1, 1)
    return conv_tensors(s, seed, "uniform")


CONFIG3_SHAPE = (GemmShape(16384, 64, 256), GemmShape(16384, 128, 64))


def config3(seed: int = 3, M: int = 16384) -> Dict[str, np.ndarray]:
    """b2b GEMM: A[Mx256], W0[256x64], W1[64x128] row-major, b0[64], b1[128], U[-0.5,0.5]."""
    return dict(A=uniform_fp16(seed, 0, (M, 256), -0.5, 0.5),
                W0=uniform_fp16(seed, 1, (256, 64), -0.5, 0.5),
                b0=uniform_fp16(seed, 2, (64,), -0.5, 0.5),
                W1=uniform_fp16(seed, 3, (64, 128), -0.5, 0.5),
                b1=uniform_fp16(seed, 4, (128,), -0.5, 0.5))


CONFIG4_SHAPES = (ConvShape(32, 56, 56, 64, 64, 3, 3, 1, 1), ConvShape(32, 56, 56, 64, 256, 1, 1, 1, 0))


def config4(seed: int = 4, batch: int = 32) -> Dict[str, np.ndarray]:
    """b2b conv: 3x3 64->64 pad 1 then 1x1 64->256; weights N(0, 2/fan_in); x, biases U[-1,1]."""
    s0 = ConvShape(batch, 56, 56, 64, 64, 3, 3, 1, 1)
    s1 = ConvShape(batch, 56, 56, 64, 256, 1, 1, 1, 0)
    t0 = conv_tensors(s0, seed, "normal")
    t1 = conv_tensors(s1, seed + 1000, "normal")
    return dict(x=t0["x"], w0=t0["w"], b0=t0["bias"], w1=t1["w"], b1=t1["bias"])


def config5_layer(index: int, batch: int = 32) -> Tuple[ConvShape, int, Dict[str, np.ndarray]]:
    """Layer `index` (0..22) of the ResNet-50-shaped stack: shape, multiplicity, unpadded tensors."""
    shape, cnt = resnet50_layers(batch)[index]
    return shape, cnt, conv_tensors(shape, 500 + index, "normal")


# Extra shapes from the paper's tables (synthetic stand-ins for its recommendation-model and
# RepVGG workloads).
TABLE1_B2B_GEMM = [  # (M, N0, K0, N1)  with K1 = N0
    (2464, 1, 4, 4), (16384, 64, 256, 16), (32768, 128, 576, 64), (128320, 32, 96, 96)]
TABLE2_B2B_CONV = [  # (H, IC, OC0, stride, OC1)
    (224, 3, 48, 2, 48), (112, 48, 48, 2, 48), (56, 48, 48, 1, 48),
    (224, 3, 64, 2, 64), (112, 64, 64, 2, 64), (56, 64, 64, 1, 64)]
EPILOGUE_GEMM = GemmShape(1280, 3072, 768)
TABLE3_PADDING = [  # (N, H, W, IC, OC, R, S, pad): stride 1, IC not divisible by 8
    (32, 20, 26, 46, 32, 3, 3, 1), (32, 20, 26, 46, 32, 5, 5, 2), (128, 14, 19, 46, 32, 5, 7, 0),
    (288, 11, 15, 46, 32, 5, 7, 0), (32, 20, 26, 174, 64, 3, 3, 1), (32, 20, 26, 174, 64, 5, 5, 2)]
