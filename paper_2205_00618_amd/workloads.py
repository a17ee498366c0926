"""Seeded synthetic inputs for the dense contractions (no arithmetic of the method here).

The generalised contraction of Section 2.1 is instantiated three ways: fp32 GEMM
(Fig. 1), 2-D convolution (first item of the list that follows the pre/post-operation
formula) and a signed 8-bit GEMM with 32-bit sums.  Table 1 of the evaluation lists the
operator shapes (MM-64..512, CONV-1..4); the shapes below follow the same pattern and
add larger and ragged ones.  All values come from ``numpy.random.default_rng(seed)``,
drawn A (or input) first, then B (or filter), and are cast to the storage type.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class GemmShape:
    M: int
    N: int
    K: int


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

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1


@dataclass(frozen=True)
class DwConvShape:
    """Depth-wise convolution: C channels, one R x S filter per channel."""
    N: int
    H: int
    W: int
    C: int
    R: int
    S: int
    stride: int
    pad: int

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def bytes(self) -> int:
        """One read of input and filter, one write of the output."""
        return 4 * (self.N * self.H * self.W * self.C + self.R * self.S * self.C
                    + self.N * self.P * self.Q * self.C)


# The five named workloads: (seed, shapes).
SGEMM_SMALL = (0, GemmShape(64, 64, 64))
SGEMM_4096 = (1, GemmShape(4096, 4096, 4096))
SGEMM_RAGGED = (2, [GemmShape(1000, 1000, 1000), GemmShape(4096, 4096, 256),
                    GemmShape(256, 256, 8192), GemmShape(4097, 129, 511)])
CONV_56 = (3, ConvShape(32, 56, 56, 64, 64, 3, 3, 1, 1))
IGEMM_1024 = (4, GemmShape(1024, 1024, 1024))

# Operator shapes of Table 1 (matrix multiplications and 3x3 stride-1 convolutions).
TABLE1_MM = [GemmShape(n, n, n) for n in (64, 128, 256, 512)]
# Depth-wise rows of Table 1 (DWCONV-1..4): channels, image size, filter, stride; "same"
# padding (R // 2) and the batch are this library's choice, the table gives neither.
def table1_dwconv(batch: int = 1):
    return [DwConvShape(batch, 112, 112, 16, 3, 3, 2, 1), DwConvShape(batch, 56, 56, 72, 3, 3, 2, 1),
            DwConvShape(batch, 28, 28, 88, 3, 3, 1, 1), DwConvShape(batch, 14, 14, 240, 5, 5, 1, 2)]


TABLE1_DWCONV_SEED = 5
TABLE1_CONV = [ConvShape(1, 56, 56, 64, 128, 3, 3, 1, 0), ConvShape(1, 28, 28, 128, 256, 3, 3, 1, 0),
               ConvShape(1, 14, 14, 256, 512, 3, 3, 1, 0), ConvShape(1, 7, 7, 512, 512, 3, 3, 1, 0)]


def uniform_f32(rng: np.random.Generator, shape, lo=-1.0, hi=1.0) -> np.ndarray:
    return rng.uniform(lo, hi, size=shape).astype(np.float32)


def small_int_f32(rng: np.random.Generator, shape, bound=8) -> np.ndarray:
    """Integers in [-bound, bound] stored as fp32: sums stay exactly representable."""
    return rng.integers(-bound, bound + 1, size=shape).astype(np.float32)


def sgemm_inputs(seed: int, shape: GemmShape, exact: bool = False,
                 c_zero: bool = True) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """A (MxK), B (KxN), C (MxN), row-major and tightly strided."""
    rng = np.random.default_rng(seed)
    return sgemm_inputs_from(rng, shape, exact, c_zero)


def sgemm_inputs_from(rng, shape: GemmShape, exact: bool = False, c_zero: bool = True):
    draw = small_int_f32 if exact else uniform_f32
    A = draw(rng, (shape.M, shape.K))
    B = draw(rng, (shape.K, shape.N))
    C = np.zeros((shape.M, shape.N), np.float32) if c_zero else draw(rng, (shape.M, shape.N))
    return A, B, C


def sgemm_ragged_inputs(seed: int = SGEMM_RAGGED[0], shapes: List[GemmShape] = SGEMM_RAGGED[1]):
    """The rectangular / edge shapes, all drawn in listed order from one generator."""
    rng = np.random.default_rng(seed)
    return [(s,) + sgemm_inputs_from(rng, s) for s in shapes]


def conv_inputs(seed: int, shape: ConvShape, exact: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """Input NHWC in [0,1) (post-activation-like) and filter KRSC ~ normal(0, 0.1)."""
    rng = np.random.default_rng(seed)
    if exact:
        x = rng.integers(0, 5, size=(shape.N, shape.H, shape.W, shape.C)).astype(np.float32)
        w = rng.integers(-4, 5, size=(shape.K, shape.R, shape.S, shape.C)).astype(np.float32)
    else:
        x = rng.random(size=(shape.N, shape.H, shape.W, shape.C)).astype(np.float32)
        w = rng.normal(0.0, 0.1, size=(shape.K, shape.R, shape.S, shape.C)).astype(np.float32)
    return x, w


def dwconv_inputs(seed: int, shape: DwConvShape, exact: bool = False):
    """Input NHWC in [0,1), filter RSC ~ normal(0, 0.1), bias (C) ~ normal(0, 0.1)."""
    rng = np.random.default_rng(seed)
    xs, ws = (shape.N, shape.H, shape.W, shape.C), (shape.R, shape.S, shape.C)
    if exact:
        x = rng.integers(0, 5, size=xs).astype(np.float32)
        w = rng.integers(-4, 5, size=ws).astype(np.float32)
        bias = rng.integers(-20, 21, size=shape.C).astype(np.float32)
    else:
        x = rng.random(size=xs).astype(np.float32)
        w = rng.normal(0.0, 0.1, size=ws).astype(np.float32)
        bias = rng.normal(0.0, 0.1, size=shape.C).astype(np.float32)
    return x, w, bias


def igemm_inputs(seed: int, shape: GemmShape, c_zero: bool = True):
    """Signed 8-bit A (MxK), B (KxN) uniform over [-128, 127]; C int32."""
    rng = np.random.default_rng(seed)
    A = rng.integers(-128, 128, size=(shape.M, shape.K), dtype=np.int8)
    B = rng.integers(-128, 128, size=(shape.K, shape.N), dtype=np.int8)
    if c_zero:
        C = np.zeros((shape.M, shape.N), np.int32)
    else:
        C = rng.integers(-2**20, 2**20, size=(shape.M, shape.N), dtype=np.int32)
    return A, B, C


def with_ld(a: np.ndarray, ld: int, fill=0) -> np.ndarray:
    """Copy a 2-D array into a buffer whose rows are ``ld`` elements apart; returns the
    padded buffer (rows x ld); the payload is ``buf[:, :a.shape[1]]``."""
    rows, cols = a.shape
    assert ld >= cols
    buf = np.full((rows, ld), fill, dtype=a.dtype)
    buf[:, :cols] = a
    return buf


def sample_points(seed: int, M: int, N: int, count: int, tile: int = 128):
    """Output coordinates for spot checks: uniform samples plus the corners and the
    last row/column of tiles, where indexing mistakes show first."""
    rng = np.random.default_rng(seed)
    ii = rng.integers(0, M, size=count)
    jj = rng.integers(0, N, size=count)
    edge_i = [0, M - 1, min(tile - 1, M - 1), min(tile, M - 1), (M - 1) // tile * tile]
    edge_j = [0, N - 1, min(tile - 1, N - 1), min(tile, N - 1), (N - 1) // tile * tile]
    ei, ej = np.meshgrid(edge_i, edge_j, indexing="ij")
    ii = np.concatenate([ii, ei.ravel()]).astype(np.int64)
    jj = np.concatenate([jj, ej.ravel()]).astype(np.int64)
    return ii, jj
