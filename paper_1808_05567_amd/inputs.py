"""Seeded synthetic inputs and the workload shapes.

This module holds no convolution arithmetic.  It is the one piece shared by
the GPU tests/benchmark and the CPU oracle's tests: both sides are fed the
very same host-generated numbers.

Shapes are the 20 ResNet-50 convolution layers of Table I of the paper
(C, K, H, W, R, S, stride).  The table has no padding column; the pads used
here are the ResNet-50 ones (7x7 -> 3, 3x3 -> 1, 1x1 -> 0).

A second workload, the distinct convolution shapes of Inception-v3 at 299 x 299
(the paper reports layer averages for it in Section III-A but prints no layer
list; the shapes below are those of the public model definition, each listed
once), brings rectangular 1x7 / 7x1 / 1x3 / 3x1 filters padded along their long
side only, a 5x5 filter and unpadded stride-2 3x3 filters.

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
    pad_h: int = -1   # -1: "same"-style padding, (R-1)/2 rows and (S-1)/2 columns
    pad_w: int = -1

    @property
    def pads(self):
        return ((self.R - 1) // 2 if self.pad_h < 0 else self.pad_h,
                (self.S - 1) // 2 if self.pad_w < 0 else self.pad_w)

    @property
    def pad(self):
        """One int where both axes are padded alike, else the pair (pad_h, pad_w)."""
        ph, pw = self.pads
        return ph if ph == pw else (ph, pw)

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pads[0] - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pads[1] - self.S) // self.stride + 1

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




def _v3():
    rows = []

    def add(C, K, HW, R, S, stride=1, valid=False):
        rows.append(Layer(len(rows) + 1, C, K, HW, HW, R, S, stride,
                          0 if valid else -1, 0 if valid else -1))

    # stem
    add(3, 32, 299, 3, 3, 2, valid=True)
    add(32, 32, 149, 3, 3, valid=True)
    add(32, 64, 147, 3, 3)
    add(64, 80, 73, 1, 1)
    add(80, 192, 73, 3, 3, valid=True)
    # 35 x 35 modules (inputs of 192, 256, 288 channels)
    for cin in (192, 256, 288):
        add(cin, 64, 35, 1, 1)
        add(cin, 48, 35, 1, 1)
        if cin == 192:
            add(cin, 32, 35, 1, 1)
    add(48, 64, 35, 5, 5)
    add(64, 96, 35, 3, 3)
    add(96, 96, 35, 3, 3)
    # grid reduction 35 -> 17
    add(288, 384, 35, 3, 3, 2, valid=True)
    add(96, 96, 35, 3, 3, 2, valid=True)
    # 17 x 17 modules with factorised 7x7 filters (branch widths 128, 160, 192)
    add(768, 192, 17, 1, 1)
    for c7 in (128, 160, 192):
        if c7 != 192:
            add(768, c7, 17, 1, 1)
            add(c7, c7, 17, 1, 7)
            add(c7, c7, 17, 7, 1)
        add(c7, 192, 17, 1, 7)
        add(c7, 192, 17, 7, 1)
    # grid reduction 17 -> 8
    add(192, 320, 17, 3, 3, 2, valid=True)
    add(192, 192, 17, 3, 3, 2, valid=True)
    # 8 x 8 modules with 1x3 / 3x1 pairs (inputs of 1280 and 2048 channels)
    for cin in (1280, 2048):
        for k in (320, 384, 448, 192):
            add(cin, k, 8, 1, 1)
    add(384, 384, 8, 1, 3)
    add(384, 384, 8, 3, 1)
    add(448, 384, 8, 3, 3)
    return tuple(rows)


# Distinct convolution shapes of Inception-v3 (299 x 299 input), ids 1..len.
INCEPTION_V3 = _v3()

WORKLOADS = {"resnet50": TABLE_I, "inception_v3": INCEPTION_V3}


def layer(layer_id: int, workload: str = "resnet50") -> Layer:
    return WORKLOADS[workload][layer_id - 1]


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
