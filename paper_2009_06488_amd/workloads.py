"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random codes and constants; it holds none of the
method's arithmetic (no packing, no products, no re-quantization) so that the
GPU library and the CPU oracle can both be fed from it without sharing code.

Codes are uint8 arrays with one 4-bit code (0..15, all sixteen equally likely)
per byte, except for the large GEMM, which draws packed bytes directly (a
uniform random byte is two independent uniform codes).

The paper times randomly initialised matrices whose sizes are those of compact
CNN layers (Sec. 4.1) and a small OCR CNN (Sec. 4.2, Table 2); the shapes below
keep that kind (depths that are 3x3xC im2col depths) at the sizes the benchmark
configuration names.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np


def _codes(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.integers(0, 16, size=shape, dtype=np.uint8)


@dataclass
class GemmCase:
    name: str
    M: int
    N: int
    K: int
    za: int
    zb: int
    seed: int
    a_codes: np.ndarray = None   # M x K, one code per byte
    b_codes: np.ndarray = None   # K x N, one code per byte


def gemm_case(name: str, M: int, N: int, K: int, seed: int, za=None, zb=None) -> GemmCase:
    """Draw order: za, zb (only when not given), A codes, B codes."""
    rng = np.random.default_rng(seed)
    if za is None:
        za = int(rng.integers(0, 16))
    if zb is None:
        zb = int(rng.integers(0, 16))
    a = _codes(rng, (M, K))
    b = _codes(rng, (K, N))
    return GemmCase(name, M, N, K, int(za), int(zb), seed, a, b)


def config1() -> GemmCase:
    """Single small GEMM: 64 x 72 times 72 x 32, za=7, zb=8, seed 0."""
    return gemm_case("cfg1_64x32x72", 64, 32, 72, seed=0, za=7, zb=8)


def config2_shapes() -> List[Tuple[int, int, int, int]]:
    """(M, N, K, seed) of the 27-case sweep; zero points are drawn per case."""
    out = []
    i = 0
    for M in (64, 256, 1024):
        for N in (64, 256, 1024):
            for K in (72, 288, 1152):
                out.append((M, N, K, 2000 + i))
                i += 1
    return out


def config2() -> List[GemmCase]:
    return [gemm_case(f"cfg2_{M}x{N}x{K}", M, N, K, seed) for (M, N, K, seed) in config2_shapes()]


@dataclass
class ConvCase:
    name: str
    N: int
    H: int
    W: int
    C: int
    KH: int
    KW: int
    stride: Tuple[int, int]
    pad: Tuple[int, int]
    OC: int
    zx: int
    zw: int
    mult: int
    shift: int
    zo: int
    seed: int
    x_codes: np.ndarray = None   # N x H x W x C
    w_codes: np.ndarray = None   # OC x KH x KW x C

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.pad[0] - self.KH) // self.stride[0] + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pad[1] - self.KW) // self.stride[1] + 1

    @property
    def depth(self) -> int:
        return self.KH * self.KW * self.C


def conv_case(name, N, H, W, C, KH, KW, stride, pad, OC, zx, zw, shift, zo, seed) -> ConvCase:
    """Draw order: x codes, w codes, multiplier in [2**14, 2**15)."""
    rng = np.random.default_rng(seed)
    x = _codes(rng, (N, H, W, C))
    w = _codes(rng, (OC, KH, KW, C))
    mult = int(rng.integers(2 ** 14, 2 ** 15))
    return ConvCase(name, N, H, W, C, KH, KW, tuple(stride), tuple(pad), OC, zx, zw, mult, shift, zo, seed, x, w)


def config3() -> ConvCase:
    """One 3x3 conv layer, 64x64x32 input, 64 output channels, pad 1, then re-quantization."""
    return conv_case("cfg3_conv64x64x32_oc64", 1, 64, 64, 32, 3, 3, (1, 1), (1, 1), 64,
                     zx=7, zw=8, shift=20, zo=8, seed=3000)


@dataclass
class CnnLayer:
    cin: int
    cout: int
    zw: int
    mult: int
    shift: int
    zo: int
    pool_after: bool
    w_codes: np.ndarray = None   # cout x 3 x 3 x cin


@dataclass
class CnnCase:
    name: str
    batch: int
    H: int
    W: int
    zx: int
    pad: int
    seed: int
    x_codes: np.ndarray = None   # batch x H x W x 1
    layers: List[CnnLayer] = field(default_factory=list)


CNN_CHANNELS = (16, 32, 32, 64, 64, 128)
CNN_SHIFTS = (18, 20, 22, 22, 22, 22)
CNN_POOL_AFTER = (False, True, False, True, False, False)


def config4(batch: int = 64, H: int = 32, W: int = 128, pad: int = 1, seed: int = 4000) -> CnnCase:
    """OCR-style CNN: six 3x3 convs 1-16-32-32-64-64-128, 2x2 max-pool after layers 2 and 4.

    Draw order: input codes, then for each layer its weight codes and its multiplier.
    """
    rng = np.random.default_rng(seed)
    case = CnnCase(f"cfg4_ocr_cnn_b{batch}", batch, H, W, zx=7, pad=pad, seed=seed)
    case.x_codes = _codes(rng, (batch, H, W, 1))
    cin = 1
    for cout, shift, pool in zip(CNN_CHANNELS, CNN_SHIFTS, CNN_POOL_AFTER):
        w = _codes(rng, (cout, 3, 3, cin))
        mult = int(rng.integers(2 ** 14, 2 ** 15))
        case.layers.append(CnnLayer(cin, cout, zw=8, mult=mult, shift=shift, zo=8, pool_after=pool, w_codes=w))
        cin = cout
    return case


@dataclass
class PackedGemmCase:
    name: str
    M: int
    N: int
    K: int
    za: int
    zb: int
    seed: int
    a_packed: np.ndarray = None   # M x K/2 bytes
    b_packed_kn: np.ndarray = None  # K x N/2 bytes


def config5(M: int = 8192, N: int = 8192, K: int = 8192, seed: int = 5000) -> PackedGemmCase:
    """Large GEMM for the roofline; draws packed bytes directly (M, N, K even)."""
    assert K % 2 == 0 and N % 2 == 0
    rng = np.random.default_rng(seed)
    a = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    b = rng.integers(0, 256, size=(K, N // 2), dtype=np.uint8)
    return PackedGemmCase(f"cfg5_{M}x{N}x{K}", M, N, K, 7, 8, seed, a, b)


# The paper's own OCR network (Table 2): six valid convolutions on a 25 x 33 grayscale input,
# (filters, kernel, stride) per layer, ReLU after each (expressed as qmin = zo in the re-quantization).
PAPER_CNN_LAYERS = ((8, 5, 1), (8, 3, 1), (8, 3, 2), (16, 3, 1), (16, 3, 2), (24, 3, 1))
PAPER_CNN_SHIFTS = (19, 19, 18, 18, 19, 19)


@dataclass
class PaperCnnLayer:
    cin: int
    cout: int
    k: int
    stride: int
    zw: int
    mult: int
    shift: int
    zo: int
    w_codes: np.ndarray = None   # cout x k x k x cin


def paper_cnn(batch: int = 8, seed: int = 4100):
    """Random-weight instance of the paper's topology; returns (x_codes batch x 25 x 33 x 1, zx, layers)."""
    rng = np.random.default_rng(seed)
    x = _codes(rng, (batch, 25, 33, 1))
    layers, cin = [], 1
    for (cout, k, stride), shift in zip(PAPER_CNN_LAYERS, PAPER_CNN_SHIFTS):
        w = _codes(rng, (cout, k, k, cin))
        mult = int(rng.integers(2 ** 14, 2 ** 15))
        layers.append(PaperCnnLayer(cin, cout, k, stride, zw=8, mult=mult, shift=shift, zo=4, w_codes=w))
        cin = cout
    return x, 7, layers
