"""GPU parity of ac_gemm_i8_static, the entry point for callers that cannot allocate: its K-slice partial sums go
through a buffer inside the library.  Checked through the C ABI against ac_gemm_i8 with a caller workspace (and
against the CPU oracle), bit for bit, on two calls in a row that share the buffer, the second on a smaller problem
whose partial sums overwrite only the start of what the first one left behind."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu

# (M, N, K): each is cut along K by the library's own plan, so each goes through the buffer
FIRST = (49, 2048, 4608)   # 8 slices, 3.2 MB of partial sums
SECOND = (24, 1024, 4608)  # 8 slices, 0.8 MB


def with_workspace(A, B, bias, shift, act):
    M, K = A.shape
    N = B.shape[1]
    nbytes = ops.ac_gemm_i8_workspace_bytes(M, N, K)
    assert nbytes > 0
    ws = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device="cuda")
    C = torch.full((M, N), 77, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8(A, B, bias, C, shift, act, workspace=ws)
    return C


def test_two_calls_in_a_row_share_the_buffer():
    assert ops.ac_gemm_i8_auto_plan(*FIRST, True)[1] > 1 and ops.ac_gemm_i8_auto_plan(*SECOND, True)[1] > 1
    assert ops.ac_gemm_i8_workspace_bytes(*SECOND) < ops.ac_gemm_i8_workspace_bytes(*FIRST) <= ops.AC_STATIC_SCRATCH_BYTES
    cases = []
    for i, (M, N, K) in enumerate((FIRST, SECOND)):
        A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=7700 + i)
        cases.append((A, B, bias, dev(A), dev(B), dev(bias), torch.full((M, N), 55, dtype=torch.int8, device="cuda")))
    shift, act = 10, ops.AC_ACT_RELU
    # the two calls follow each other on one stream with nothing in between
    for (_, _, _, dA, dB, dbias, C) in cases:
        ops.ac_gemm_i8_static(dA, dB, dbias, C, shift, act)
    torch.cuda.synchronize()
    for (A, B, bias, dA, dB, dbias, C) in cases:
        want = with_workspace(dA, dB, dbias, shift, act)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(C), host(want))
        np.testing.assert_array_equal(host(C), oracle.gemm_i8(A, B, bias, shift, act))


def test_uncut_shapes_and_refusals():
    # a shape the library does not cut runs without touching the buffer
    A, B, bias = inputs.gemm_i8_inputs(256, 256, 256, seed=7710)
    assert ops.ac_gemm_i8_workspace_bytes(256, 256, 256) == 0
    C = torch.full((256, 256), 55, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8_static(dev(A), dev(B), dev(bias), C, 8, ops.AC_ACT_NONE)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C), oracle.gemm_i8(A, B, bias, 8, ops.AC_ACT_NONE))
    # partial sums beyond the buffer: refused, nothing launched, C untouched
    M, N, K = 1024, 1024, 65536
    assert ops.ac_gemm_i8_workspace_bytes(M, N, K) > ops.AC_STATIC_SCRATCH_BYTES
    A = torch.zeros((M, K), dtype=torch.int8, device="cuda")
    B = torch.zeros((K, N), dtype=torch.int8, device="cuda")
    C = torch.full((M, N), 55, dtype=torch.int8, device="cuda")
    with pytest.raises(ops.AcError) as err:
        ops.ac_gemm_i8_static(A, B, None, C, 8, ops.AC_ACT_NONE)
    assert err.value.status == ops.AC_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((C == 55).all())
