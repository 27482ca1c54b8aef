"""Seeded synthetic inputs and the workload shapes.

This module holds no convolution arithmetic.  It is the one piece shared by
the GPU tests/benchmark and the CPU oracle's tests: both sides are fed the
very same host-generated numbers.

Shapes are the 20 ResNet-50 convolution layers of Table I of the paper
(C, K, H, W, R, S, stride).  The table has no padding column; the pads used
here are the ResNet-50 ones (7x7 -> 3, 3x3 -> 1, 1x1 -> 0).

Distributions (the paper's layer benchmark also runs on auto-generated data,
Artifact Description, "Datasets"): input and output gradient uniform on
[-1, 1), weights normal with standard deviation sqrt(2 / (C R S)).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_BASE = 180805567


@dataclass(frozen=True)
class Layer:
    id: int
    C: int
    K: int
    H: int
    W: int
    R: int
    S: int
    stride: int

    @property
    def pad(self) -> int:
        return (self.R - 1) // 2

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    def flops(self, N: int) -> int:
        """2 N K C P Q R S -- the same count for each of the three passes."""
        return 2 * N * self.K * self.C * self.P * self.Q * self.R * self.S


# Table I ("ResNet-50 layers specifications"): id, C, K, H, W, R, S, stride.
TABLE_I = (
    Layer(1, 3, 64, 224, 224, 7, 7, 2),
    Layer(2, 64, 256, 56, 56, 1, 1, 1),
    Layer(3, 64, 64, 56, 56, 1, 1, 1),
    Layer(4, 64, 64, 56, 56, 3, 3, 1),
    Layer(5, 256, 64, 56, 56, 1, 1, 1),
    Layer(6, 256, 512, 56, 56, 1, 1, 2),
    Layer(7, 256, 128, 56, 56, 1, 1, 2),
    Layer(8, 128, 128, 28, 28, 3, 3, 1),
    Layer(9, 128, 512, 28, 28, 1, 1, 1),
    Layer(10, 512, 128, 28, 28, 1, 1, 1),
    Layer(11, 512, 1024, 28, 28, 1, 1, 2),
    Layer(12, 512, 256, 28, 28, 1, 1, 2),
    Layer(13, 256, 256, 14, 14, 3, 3, 1),
    Layer(14, 256, 1024, 14, 14, 1, 1, 1),
    Layer(15, 1024, 256, 14, 14, 1, 1, 1),
    Layer(16, 1024, 2048, 14, 14, 1, 1, 2),
    Layer(17, 1024, 512, 14, 14, 1, 1, 2),
    Layer(18, 512, 512, 7, 7, 3, 3, 1),
    Layer(19, 512, 2048, 7, 7, 1, 1, 1),
    Layer(20, 2048, 512, 7, 7, 1, 1, 1),
)

LAYERS_3X3 = tuple(l for l in TABLE_I if l.R == 3)
LAYERS_1X1 = tuple(l for l in TABLE_I if l.R == 1)


def layer(layer_id: int) -> Layer:
    return TABLE_I[layer_id - 1]


def _rng(seed: int, layer_id: int, which: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=SEED_BASE + 1000 * layer_id + which
                                                + 7919 * seed))


def gen_input(N, C, H, W, layer_id=0, seed=0) -> np.ndarray:
    """I[N,C,H,W], fp32, uniform on [-1, 1)."""
    r = _rng(seed, layer_id, 0)
    a = r.random((N, C, H, W), dtype=np.float32)
    a *= 2.0
    a -= 1.0
    return a


def gen_weights(K, C, R, S, layer_id=0, seed=0) -> np.ndarray:
    """W[K,C,R,S], fp32, normal(0, sqrt(2/(C R S)))."""
    r = _rng(seed, layer_id, 1)
    a = r.standard_normal((K, C, R, S), dtype=np.float32)
    a *= np.float32(np.sqrt(2.0 / (C * R * S)))
    return a


def gen_outgrad(N, K, P, Q, layer_id=0, seed=0) -> np.ndarray:
    """dO[N,K,P,Q], fp32, uniform on [-1, 1)."""
    r = _rng(seed, layer_id, 2)
    a = r.random((N, K, P, Q), dtype=np.float32)
    a *= 2.0
    a -= 1.0
    return a


def gen_small_ints(shape, lo, hi, layer_id=0, seed=0, which=3) -> np.ndarray:
    """Integer-valued fp32 data in [lo, hi]: sums stay exact in fp32 while small."""
    r = _rng(seed, layer_id, which)
    return r.integers(lo, hi + 1, size=shape).astype(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 -> bf16 (nearest, ties to even); result returned as fp32 values.

    A data-format conversion, applied once on the host so that the oracle and
    the GPU path start from identical bf16-representable numbers.
    """
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    out = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return out.view(np.float32).reshape(a.shape)
