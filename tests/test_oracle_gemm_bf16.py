"""Pins for the bf16 GEMM oracle (Fig. 2 contraction in fp64 on exactly widened bf16 inputs)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_18574_amd import inputs


def test_bf16_widening_is_exact():
    bits = np.array([0x0000, 0x8000, 0x3F80, 0xBF80, 0x4000, 0x3F81, 0x0080, 0x7F7F, 0x0001, 0x4049], dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(oracle.bf16_to_double(bits), want)
    assert oracle.bf16_to_double(np.array([0x3F80], np.uint16))[0] == 1.0
    assert oracle.bf16_to_double(np.array([0x4049], np.uint16))[0] == 3.140625


@pytest.mark.parametrize("M,N,K", [(17, 33, 65), (64, 64, 256), (5, 130, 7)])
def test_vs_numpy_float64_matmul(M, N, K):
    A, B = inputs.gemm_bf16_inputs(M, N, K, seed=31)
    Ad = inputs.bf16_bits_to_f32(A).astype(np.float64)
    Bd = inputs.bf16_bits_to_f32(B).astype(np.float64)
    got = oracle.gemm_bf16(A, B)
    want = Ad @ Bd
    assert np.linalg.norm(got - want) / np.linalg.norm(want) < 1e-14
    # alpha / beta
    Cin = np.random.default_rng(1).standard_normal((M, N)).astype(np.float32)
    got = oracle.gemm_bf16(A, B, alpha=-1.5, beta=0.25, C_in=Cin)
    want = -1.5 * (Ad @ Bd) + 0.25 * Cin.astype(np.float64)
    assert np.linalg.norm(got - want) / np.linalg.norm(want) < 1e-14
    # sampled form
    rng = np.random.default_rng(2)
    r, c = rng.integers(0, M, 50), rng.integers(0, N, 50)
    vals, mags = oracle.gemm_bf16_at(A, B, r, c, alpha=-1.5, beta=0.25, C_in=Cin)
    np.testing.assert_array_equal(vals, got[r, c])
    np.testing.assert_allclose(mags, (np.abs(Ad)[r] * np.abs(Bd).T[c]).sum(axis=1), rtol=1e-12)


def test_exact_cases():
    rng = np.random.default_rng(3)
    # small integers: every partial sum is exactly representable, any order gives the same result
    Ai = rng.integers(-8, 9, size=(12, 40))
    Bi = rng.integers(-8, 9, size=(40, 9))
    A = inputs.f32_to_bf16_bits(Ai.astype(np.float32))
    B = inputs.f32_to_bf16_bits(Bi.astype(np.float32))
    np.testing.assert_array_equal(oracle.gemm_bf16(A, B), (Ai @ Bi).astype(np.float64))
    # identity
    _, Bn = inputs.gemm_bf16_inputs(16, 21, 16, seed=32)
    eye = inputs.f32_to_bf16_bits(np.eye(16, dtype=np.float32))
    np.testing.assert_array_equal(oracle.gemm_bf16(eye, Bn), inputs.bf16_bits_to_f32(Bn).astype(np.float64))
    # K = 1: an outer product
    a, b = inputs.gemm_bf16_inputs(7, 5, 1, seed=33)
    want = inputs.bf16_bits_to_f32(a).astype(np.float64) * inputs.bf16_bits_to_f32(b).astype(np.float64)
    np.testing.assert_array_equal(oracle.gemm_bf16(a, b), want)
    # alpha = 0: C = beta * C_in exactly
    Cin = rng.standard_normal((7, 5)).astype(np.float32)
    np.testing.assert_array_equal(oracle.gemm_bf16(a, b, alpha=0.0, beta=2.0, C_in=Cin), 2.0 * Cin.astype(np.float64))
    # transposition identity
    A, B = inputs.gemm_bf16_inputs(9, 11, 13, seed=34)
    np.testing.assert_allclose(oracle.gemm_bf16(np.ascontiguousarray(B.T), np.ascontiguousarray(A.T)),
                               oracle.gemm_bf16(A, B).T, rtol=1e-13, atol=1e-13)
