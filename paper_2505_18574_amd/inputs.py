"""Seeded synthetic inputs for the dense tensor workloads of arxiv 2505.18574.

This module is the single source of inputs for both the GPU library and the CPU
oracle.  It holds no arithmetic of the operations themselves: only shapes,
random draws and the float32 -> bfloat16 rounding of input data.

The shapes stand in for the paper's workloads, none of which ships with it:
ResNet-50 GEMM and convolution layers on the int8 accelerator (Sections 4.4.1
and 4.4.2), the 4096^3 GEMM of the GPU study (Appendix A, Table 5) and the
12x12 fine-grained linear algebra of the TinyMPC study (Section 4.4.3,
Appendix D.2).  Values are uniform int8 / int32 / [-1,1) fp32 or N(0,1).

Seeds: the 256^3 GEMM uses seed 0; every other case uses
1000 * workload_index + case_index.  Draw order is fixed per generator and is
part of the recipe (A, B, bias | in, w, bias | A, B | A, B, x, d).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

ACT_NONE = 0
ACT_RELU = 1


# ----------------------------------------------------------------------------
# workload tables
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class GemmI8Case:
    name: str
    M: int
    N: int
    K: int
    shift: int
    act: int
    seed: int

    @property
    def ops(self) -> int:
        return 2 * self.M * self.N * self.K

    @property
    def bytes(self) -> int:  # each operand read once, output written once
        return self.M * self.K + self.K * self.N + 4 * self.N + self.M * self.N


@dataclass(frozen=True)
class ConvI8Case:
    name: str
    Nb: int
    H: int
    W: int
    Cin: int
    Cout: int
    KH: int
    KW: int
    stride: int
    pad: int
    shift: int
    act: int
    seed: int

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.pad - self.KH) // self.stride + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pad - self.KW) // self.stride + 1

    @property
    def gemm_mnk(self):
        return self.Nb * self.OH * self.OW, self.Cout, self.KH * self.KW * self.Cin

    @property
    def ops(self) -> int:  # implicit-GEMM count, padding taps included
        m, n, k = self.gemm_mnk
        return 2 * m * n * k

    @property
    def bytes(self) -> int:  # NHWC input once (not the im2col matrix), weights, bias, output
        m, n, k = self.gemm_mnk
        return self.Nb * self.H * self.W * self.Cin + k * n + 4 * n + m * n


@dataclass(frozen=True)
class GemmBf16Case:
    name: str
    M: int
    N: int
    K: int
    seed: int

    @property
    def ops(self) -> int:
        return 2 * self.M * self.N * self.K

    @property
    def bytes(self) -> int:
        return 2 * self.M * self.K + 2 * self.K * self.N + 4 * self.M * self.N


@dataclass(frozen=True)
class BatchedF32Case:
    name: str
    batch: int
    n: int
    seed: int

    @property
    def ops(self) -> int:  # 2n^3 for the product, 2n^2 for the mat-vec, n for the add
        return self.batch * (2 * self.n ** 3 + 2 * self.n ** 2 + self.n)

    @property
    def bytes(self) -> int:  # A, B read, C written; x, d read, y written
        return self.batch * 4 * (3 * self.n * self.n + 3 * self.n)


GEMM_I8_256 = GemmI8Case("gemm_i8_256", 256, 256, 256, shift=8, act=ACT_RELU, seed=0)

GEMM_I8_SWEEP = tuple(
    GemmI8Case(f"gemm_i8_{m}x{n}x{k}", m, n, k, shift=10, act=ACT_RELU, seed=1000 * 2 + i)
    for i, (m, n, k) in enumerate(
        [(3136, 64, 576), (3136, 256, 64), (784, 512, 1152), (196, 1024, 2304), (49, 2048, 4608), (512, 768, 768)]
    )
)

CONV_I8 = (
    ConvI8Case("conv_i8_56x56_64to64_s1", 8, 56, 56, 64, 64, 3, 3, 1, 1, shift=9, act=ACT_RELU, seed=3000),
    ConvI8Case("conv_i8_28x28_128to256_s2", 8, 28, 28, 128, 256, 3, 3, 2, 1, shift=9, act=ACT_RELU, seed=3001),
)

GEMM_BF16 = (
    GemmBf16Case("gemm_bf16_4096", 4096, 4096, 4096, seed=4000),
    GemmBf16Case("gemm_bf16_8192x4096x1024", 8192, 4096, 1024, seed=4001),
)

BATCHED_F32 = BatchedF32Case("batched_f32_262144x12", 262144, 12, seed=5000)

# Shapes the paper names outside its main sweep, read as M x N x K (the order its 12544x64x256 kernel fixes:
# A[12544][256], B[256][64], Appendix D.1): the GEMM of the code example, and the square / column-dominant /
# row-dominant families of the schedule-reuse study (Section 5, Table 2: a base shape followed by its two
# reuse targets).
GEMM_I8_PAPER = tuple(
    GemmI8Case(f"gemm_i8_{m}x{n}x{k}", m, n, k, shift=10, act=ACT_RELU, seed=1000 * 6 + i)
    for i, (m, n, k) in enumerate(
        [(12544, 64, 256),
         (1024, 1024, 1024), (512, 512, 512), (256, 256, 256),
         (12544, 256, 64), (6272, 256, 64), (12544, 128, 64),
         (128, 1024, 1024), (64, 1024, 1024), (32, 1024, 1024)]
    )
)
GEMM_I8_REUSE_FAMILIES = ((1, 2, 3), (4, 5, 6), (7, 8, 9))  # indices into GEMM_I8_PAPER: base, target, target

# GEMM shapes of the accelerator and GPU studies (Appendix A, Tables 3 and 5), written there as
# (M x K) * (K x N): a tall-K product, the 4096 x 8192 x 8192 GEMM, a very deep K and a very shallow K.
GEMM_BF16_PAPER = tuple(
    GemmBf16Case(f"gemm_bf16_{m}x{n}x{k}", m, n, k, seed=1000 * 7 + i)
    for i, (m, n, k) in enumerate(
        [(2048, 4096, 8192), (4096, 8192, 8192), (256, 256, 524288), (32768, 32768, 32)]
    )
)


# ----------------------------------------------------------------------------
# bf16 input rounding (data preparation, not part of any operation)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 (ties to even); returns uint16 bit patterns.

    Finite inputs only (the generators never produce NaN or infinity)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------
def _rng(seed: int) -> np.random.Generator:
    return np.random.default_rng(seed)


def gemm_i8_inputs(M: int, N: int, K: int, seed: int, lo: int = -128, hi: int = 127, bias_bits: int = 15,
                   bias_matrix: bool = False):
    """A (M,K) int8, B (K,N) int8 uniform in [lo,hi]; bias int32 uniform in [-2^bias_bits, 2^bias_bits)."""
    g = _rng(seed)
    A = g.integers(lo, hi + 1, size=(M, K), dtype=np.int64).astype(np.int8)
    B = g.integers(lo, hi + 1, size=(K, N), dtype=np.int64).astype(np.int8)
    shape = (M, N) if bias_matrix else (N,)
    bias = g.integers(-(1 << bias_bits), 1 << bias_bits, size=shape, dtype=np.int64).astype(np.int32)
    return A, B, bias


def gemm_i8_case_inputs(case: GemmI8Case):
    return gemm_i8_inputs(case.M, case.N, case.K, case.seed)


def conv_i8_inputs(Nb, H, W, Cin, Cout, KH, KW, seed, lo: int = -128, hi: int = 127, bias_bits: int = 15):
    """x (Nb,H,W,Cin) int8, w (KH,KW,Cin,Cout) int8, bias (Cout,) int32."""
    g = _rng(seed)
    x = g.integers(lo, hi + 1, size=(Nb, H, W, Cin), dtype=np.int64).astype(np.int8)
    w = g.integers(lo, hi + 1, size=(KH, KW, Cin, Cout), dtype=np.int64).astype(np.int8)
    bias = g.integers(-(1 << bias_bits), 1 << bias_bits, size=(Cout,), dtype=np.int64).astype(np.int32)
    return x, w, bias


def conv_i8_case_inputs(case: ConvI8Case):
    return conv_i8_inputs(case.Nb, case.H, case.W, case.Cin, case.Cout, case.KH, case.KW, case.seed)


def gemm_bf16_inputs(M: int, N: int, K: int, seed: int):
    """A (M,K), B (K,N): N(0,1) float32 samples rounded to bf16; returned as uint16 bit patterns."""
    g = _rng(seed)
    A = f32_to_bf16_bits(g.standard_normal(size=(M, K), dtype=np.float32))
    B = f32_to_bf16_bits(g.standard_normal(size=(K, N), dtype=np.float32))
    return A, B


def gemm_bf16_case_inputs(case: GemmBf16Case):
    return gemm_bf16_inputs(case.M, case.N, case.K, case.seed)


def batched_f32_inputs(batch: int, n: int, seed: int):
    """A, B (batch,n,n), x, d (batch,n): float32 uniform in [-1,1)."""
    g = _rng(seed)

    def u(shape):
        return (g.random(size=shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)).astype(np.float32)

    A = u((batch, n, n))
    B = u((batch, n, n))
    x = u((batch, n))
    d = u((batch, n))
    return A, B, x, d


def batched_f32_case_inputs(case: BatchedF32Case):
    return batched_f32_inputs(case.batch, case.n, case.seed)


def tinympc_inputs(batch: int, seed: int, nx: int = 12, nu: int = 4, horizon: int = 5):
    """Adyn (nx,nx), Bdyn (nx,nu), Kinf (nu,nx) shared; x0 (batch,nx), d (batch,horizon,nu): uniform [-1,1)."""
    g = _rng(seed)

    def u(shape):
        return (g.random(size=shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)).astype(np.float32)

    return u((nx, nx)), u((nx, nu)), u((nu, nx)), u((batch, nx)), u((batch, horizon, nu))
