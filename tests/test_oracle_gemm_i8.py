"""Pins for the int8 GEMM oracle (Fig. 2 contraction, Fig. 14 bias, Fig. 15 output stage)."""
import numpy as np
import pytest

import oracle
from paper_2505_18574_amd import inputs


def epilogue_np(acc, shift, relu):
    """Independent formulation: exact float64 division and numpy's half-to-even rint."""
    q = np.rint(acc.astype(np.float64) / float(1 << shift)).astype(np.int64)
    q = np.clip(q, -128, 127)
    if relu:
        q = np.maximum(q, 0)
    return q.astype(np.int8)


def brute(A, B, bias, shift, relu):
    M, K = A.shape
    N = B.shape[1]
    out = np.zeros((M, N), dtype=np.int8)
    for i in range(M):
        for j in range(N):
            s = 0
            for k in range(K):
                s += int(A[i, k]) * int(B[k, j])
            if bias is not None:
                s += int(bias[j]) if bias.ndim == 1 else int(bias[i, j])
            out[i, j] = oracle.requantise(s, shift, 1 if relu else 0)
    return out


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 4), (5, 4, 3), (3, 5, 5), (4, 2, 1)])
@pytest.mark.parametrize("shift,relu", [(0, 0), (3, 1), (8, 0)])
def test_brute_force_tiny(M, N, K, shift, relu):
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M * 100 + N * 10 + K)
    got = oracle.gemm_i8(A, B, bias, shift, relu)
    np.testing.assert_array_equal(got, brute(A, B, bias, shift, relu))
    # extremes
    A[:] = -128
    B[:] = np.where(np.arange(B.size).reshape(B.shape) % 2 == 0, 127, -128)
    np.testing.assert_array_equal(oracle.gemm_i8(A, B, None, shift, relu), brute(A, B, None, shift, relu))


@pytest.mark.parametrize("M,N,K,shift", [(33, 17, 70, 8), (64, 48, 256, 10), (7, 130, 19, 0), (50, 3, 300, 9)])
def test_vs_numpy_int64_matmul(M, N, K, shift):
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=11)
    acc = A.astype(np.int64) @ B.astype(np.int64) + bias.astype(np.int64)[None, :]
    for relu in (0, 1):
        got, acc_o = oracle.gemm_i8(A, B, bias, shift, relu, return_acc=True)
        np.testing.assert_array_equal(acc_o, acc)
        np.testing.assert_array_equal(got, epilogue_np(acc, shift, relu))
    # full-matrix bias
    A, B, biasm = inputs.gemm_i8_inputs(M, N, K, seed=12, bias_matrix=True)
    acc = A.astype(np.int64) @ B.astype(np.int64) + biasm.astype(np.int64)
    np.testing.assert_array_equal(oracle.gemm_i8(A, B, biasm, shift, 1), epilogue_np(acc, shift, 1))
    # no bias
    acc = A.astype(np.int64) @ B.astype(np.int64)
    np.testing.assert_array_equal(oracle.gemm_i8(A, B, None, shift, 0), epilogue_np(acc, shift, 0))


def test_identity_and_zero():
    _, B, bias = inputs.gemm_i8_inputs(24, 37, 24, seed=3)
    eye = np.eye(24, dtype=np.int8)
    np.testing.assert_array_equal(oracle.gemm_i8(eye, B, None, 0, 0), B)
    A0 = np.zeros((9, 24), dtype=np.int8)
    small_bias = (bias % 100).astype(np.int32)
    got = oracle.gemm_i8(A0, B, small_bias, 0, 0)
    np.testing.assert_array_equal(got, np.broadcast_to(small_bias.astype(np.int8), (9, 37)))
    # B = identity: C = A
    A, _, _ = inputs.gemm_i8_inputs(13, 20, 20, seed=4)
    np.testing.assert_array_equal(oracle.gemm_i8(A, np.eye(20, dtype=np.int8), None, 0, 0), A)
    # K = 0: the contraction is empty, the output is the stage applied to the bias
    got = oracle.gemm_i8(np.zeros((4, 0), np.int8), np.zeros((0, 37), np.int8), bias, 8, 1)
    np.testing.assert_array_equal(got, np.broadcast_to(epilogue_np(bias.astype(np.int64), 8, 1), (4, 37)))


def test_linearity_before_requantisation():
    # small values, shift 0: no clamping, so the map is linear in A, in B and additive in the bias
    A1, B, b1 = inputs.gemm_i8_inputs(16, 12, 40, seed=5, lo=-3, hi=3, bias_bits=3)
    A2, B2, b2 = inputs.gemm_i8_inputs(16, 12, 40, seed=6, lo=-3, hi=3, bias_bits=3)
    f = lambda A, B, b: oracle.gemm_i8(A, B, b, 0, 0).astype(np.int64)
    np.testing.assert_array_equal(f(A1 + A2, B, b1 + b2), f(A1, B, b1) + f(A2, B, b2))
    _, acc = oracle.gemm_i8(A1, B + B2, None, 0, 0, return_acc=True)
    _, acc1 = oracle.gemm_i8(A1, B, None, 0, 0, return_acc=True)
    _, acc2 = oracle.gemm_i8(A1, B2, None, 0, 0, return_acc=True)
    np.testing.assert_array_equal(acc, acc1 + acc2)
    assert np.abs(acc).max() <= 127  # premise: nothing was clamped above
    # transposition identity: (A B)^T = B^T A^T catches swapped operands or indices
    _, accT = oracle.gemm_i8(np.ascontiguousarray(B.T), np.ascontiguousarray(A1.T), None, 0, 0, return_acc=True)
    np.testing.assert_array_equal(accT, acc1.T)


def test_saturation_closed_forms():
    a = np.full((2, 1), -128, dtype=np.int8)
    assert oracle.gemm_i8(a, np.full((1, 3), -128, np.int8), None, 0, 0).tolist() == [[127] * 3] * 2
    assert oracle.gemm_i8(a, np.full((1, 3), 127, np.int8), None, 0, 0).tolist() == [[-128] * 3] * 2
    assert oracle.gemm_i8(a, np.full((1, 3), 127, np.int8), None, 0, 1).tolist() == [[0] * 3] * 2
    # K copies of 127*127 = 16129: shift 8 -> K*63.0039.. ; K=2 -> 126.0078 -> 126 ; K=3 -> 189 -> 127
    for K, want in ((1, 63), (2, 126), (3, 127)):
        got = oracle.gemm_i8(np.full((1, K), 127, np.int8), np.full((K, 1), 127, np.int8), None, 8, 0)
        assert got[0, 0] == want


def test_permutation_equivariance():
    A, B, bias = inputs.gemm_i8_inputs(19, 23, 31, seed=8)
    rng = np.random.default_rng(0)
    pr, pc, pk = rng.permutation(19), rng.permutation(23), rng.permutation(31)
    base = oracle.gemm_i8(A, B, bias, 9, 1)
    np.testing.assert_array_equal(oracle.gemm_i8(A[pr], B, bias, 9, 1), base[pr])
    np.testing.assert_array_equal(oracle.gemm_i8(A, B[:, pc], bias[pc], 9, 1), base[:, pc])
    np.testing.assert_array_equal(oracle.gemm_i8(A[:, pk], B[pk], bias, 9, 1), base)


def test_int32_overflow_is_reported():
    A = np.ones((1, 1), np.int8)
    B = np.ones((1, 1), np.int8)
    with pytest.raises(OverflowError):
        oracle.gemm_i8(A, B, np.array([2 ** 31 - 1], np.int32), 0, 0)
    oracle.gemm_i8(A, B, np.array([2 ** 31 - 2], np.int32), 0, 0)
    # the largest workload (K = 4608) cannot overflow: K * 2^14 + 2^15 < 2^31
    assert 4608 * (1 << 14) + (1 << 15) < 2 ** 31


def test_sampled_form_matches_full():
    A, B, bias = inputs.gemm_i8_inputs(40, 50, 60, seed=9)
    full = oracle.gemm_i8(A, B, bias, 8, 1)
    rng = np.random.default_rng(1)
    r, c = rng.integers(0, 40, 200), rng.integers(0, 50, 200)
    np.testing.assert_array_equal(oracle.gemm_i8_at(A, B, bias, 8, 1, r, c), full[r, c])


def test_workload_config_256():
    """The 256^3 workload: most outputs saturate or are cleared by ReLU, as the input statistics predict."""
    case = inputs.GEMM_I8_256
    A, B, bias = inputs.gemm_i8_case_inputs(case)
    assert bias.shape == (256,) and bias.min() >= -(1 << 15) and bias.max() < (1 << 15)
    C, acc = oracle.gemm_i8(A, B, bias, case.shift, case.act, return_acc=True)
    np.testing.assert_array_equal(C, epilogue_np(A.astype(np.int64) @ B.astype(np.int64) + bias, 8, 1))
    assert C.min() == 0 and C.max() == 127
    # accumulator standard deviation ~ sqrt(K) * 5461 (product of two uniform int8 values)
    assert 0.9 < acc.std() / (np.sqrt(256) * 5461.25) < 1.1
