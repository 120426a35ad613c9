"""GPU parity: ac_gemm_i8_t (transposed operands, Appendix C Fig. 14 A_transpose / B_transpose) against the
oracle of the untransposed product: the device gets A^T and / or B^T, the oracle gets A and B."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu

FLAGS = [(True, False), (False, True), (True, True), (False, False)]


def run(A, B, bias, shift, act, ta, tb, pad=0):
    """Launch with A^T / B^T as requested; pad > 0 embeds the operands in wider arrays (leading dimension > row)."""
    M, K = A.shape
    N = B.shape[1]
    Ah = np.ascontiguousarray(A.T) if ta else A
    Bh = np.ascontiguousarray(B.T) if tb else B

    def embed(x):
        if pad == 0:
            return dev(x)
        big = torch.zeros((x.shape[0], x.shape[1] + pad), dtype=torch.int8, device="cuda")
        view = big[:, pad // 2: pad // 2 + x.shape[1]]
        view.copy_(dev(x))
        return view

    C = torch.full((M, N), 33, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8_t(embed(Ah), embed(Bh), dev(bias), C, shift, act, trans_a=ta, trans_b=tb)
    torch.cuda.synchronize()
    return host(C)


@pytest.mark.parametrize("ta,tb", FLAGS)
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (5, 3, 7), (64, 64, 64), (70, 90, 50), (128, 144, 256), (257, 300, 129),
                                    (784, 512, 1152), (2100, 2052, 200)])
def test_shapes_bit_exact(M, N, K, ta, tb):
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + 2 * N + 3 * K)
    want = oracle.gemm_i8(A, B, bias, 9, 1)
    np.testing.assert_array_equal(run(A, B, bias, 9, 1, ta, tb), want)


# Operands the direct-to-LDS kernels take (aligned, M, N and K in whole 16-byte chunks): every square tile size,
# ragged edges, a partial last K tile, several tiles per compute unit (the persistent loop with its prefetch of
# the next tile), one K tile, a deep K
@pytest.mark.parametrize("ta,tb", FLAGS[:3])
@pytest.mark.parametrize("M,N,K", [(16, 16, 16), (64, 64, 128), (80, 112, 208), (304, 272, 4160), (2112, 2064, 208), (1024, 1024, 1024),
                                    (4096, 3072, 64), (4352, 4368, 320), (8192, 256, 576), (256, 8192, 48)])
def test_direct_to_lds_shapes(M, N, K, ta, tb):
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + 2 * N + 3 * K)
    want = oracle.gemm_i8(A, B, bias, 10, 1)
    np.testing.assert_array_equal(run(A, B, bias, 10, 1, ta, tb), want)
    np.testing.assert_array_equal(run(A, B, bias, 10, 1, ta, tb, pad=64), want)  # row pitch beyond the row


@pytest.mark.parametrize("ta,tb", FLAGS[:3])
def test_small_values_matrix_bias_and_unaligned_views(ta, tb):
    M, N, K = 100, 72, 200
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=11, lo=-4, hi=4, bias_bits=6, bias_matrix=True)
    for shift, act in ((0, 0), (3, 1)):
        want = oracle.gemm_i8(A, B, bias, shift, act)
        np.testing.assert_array_equal(run(A, B, bias, shift, act, ta, tb), want)
        np.testing.assert_array_equal(run(A, B, bias, shift, act, ta, tb, pad=6), want)    # odd base offset: byte loads
        np.testing.assert_array_equal(run(A, B, bias, shift, act, ta, tb, pad=32), want)   # aligned offset, wider pitch


def test_transposed_equals_plain_entry():
    """The same product through ac_gemm_i8 and through every flag combination of ac_gemm_i8_t."""
    case = inputs.GEMM_I8_SWEEP[5]
    A, B, bias = inputs.gemm_i8_case_inputs(case)
    C0 = torch.empty((case.M, case.N), dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8(dev(A), dev(B), dev(bias), C0, case.shift, case.act)
    torch.cuda.synchronize()
    for ta, tb in FLAGS:
        np.testing.assert_array_equal(run(A, B, bias, case.shift, case.act, ta, tb), host(C0))


def test_stride_validation():
    A = torch.zeros((32, 48), dtype=torch.int8, device="cuda")   # A^T: K = 32, M = 48
    B = torch.zeros((64, 32), dtype=torch.int8, device="cuda")   # B^T: N = 64, K = 32
    C = torch.zeros((48, 64), dtype=torch.int8, device="cuda")
    L = ops.lib()
    ok = L.ac_gemm_i8_t(A.data_ptr(), 48, B.data_ptr(), 32, None, 0, C.data_ptr(), 64, 48, 64, 32, 0, 0, 1, 1, None)
    assert ok == ops.AC_OK
    assert L.ac_gemm_i8_t(A.data_ptr(), 47, B.data_ptr(), 32, None, 0, C.data_ptr(), 64, 48, 64, 32, 0, 0, 1, 1, None) == ops.AC_ERR_STRIDE
    assert L.ac_gemm_i8_t(A.data_ptr(), 48, B.data_ptr(), 31, None, 0, C.data_ptr(), 64, 48, 64, 32, 0, 0, 1, 1, None) == ops.AC_ERR_STRIDE
    torch.cuda.synchronize()
