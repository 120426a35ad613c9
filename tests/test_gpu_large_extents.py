"""GPU parity where byte offsets leave 32 bits: outputs larger than 4 GiB (sampled rows on both sides of the
2^31 and 2^32 byte marks, checked against the oracle) and operand row pitches so long that 256 rows span more
than 4 GiB (such operands take the kernels whose lanes carry 64-bit addresses)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host, rel_fro
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu


def sample_rows(M, row_bytes, seed):
    """First and last rows, the rows next to the 2^31 and 2^32 byte offsets, and a random handful."""
    rows = {0, 1, M - 2, M - 1}
    for mark in (1 << 31, 1 << 32):
        r = mark // row_bytes
        rows.update(x for x in (r - 1, r, r + 1) if 0 <= x < M)
    rows.update(int(x) for x in np.random.default_rng(seed).integers(0, M, 24))
    return np.array(sorted(rows), dtype=np.int64)


def test_int8_output_beyond_4_gib():
    M, N, K, shift = 70000, 65536, 32, 5
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=9100)
    C = torch.full((M, N), 91, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8(dev(A), dev(B), dev(bias), C, shift, 1)
    torch.cuda.synchronize()
    rows = sample_rows(M, N, 1)
    assert rows.max() * N >= 1 << 32
    want = oracle.gemm_i8(A[rows], B, bias, shift, 1)
    np.testing.assert_array_equal(host(C[torch.from_numpy(rows).cuda()]), want)


def test_int32_accumulator_output_beyond_4_gib():
    M, N, K = 40000, 32768, 32
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=9101)
    C = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    ops.ac_gemm_i8_acc32(dev(A), dev(B), dev(bias), C)
    torch.cuda.synchronize()
    rows = sample_rows(M, 4 * N, 2)
    assert rows.max() * 4 * N >= 1 << 32
    _, want = oracle.gemm_i8(A[rows], B, bias, 0, 0, return_acc=True)
    np.testing.assert_array_equal(host(C[torch.from_numpy(rows).cuda()]).astype(np.int64), want)


def test_bf16_output_beyond_4_gib():
    M, N, K = 40000, 32768, 32
    A, B = inputs.gemm_bf16_inputs(M, N, K, seed=9102)
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ops.ac_gemm_bf16(dev(A), dev(B), C, 1.0, 0.0)
    torch.cuda.synchronize()
    rows = sample_rows(M, 4 * N, 3)
    want = oracle.gemm_bf16(A[rows], B)
    got = host(C[torch.from_numpy(rows).cuda()])
    assert rel_fro(got, want) <= 1e-3
    assert np.abs(got - want).max() <= 1e-4 * np.abs(want).max()


def strided(t2d, pitch):
    """The same matrix in rows `pitch` elements apart (the gaps are never read)."""
    rows, cols = t2d.shape
    big = torch.empty(rows * pitch, dtype=t2d.dtype, device="cuda")
    view = big.as_strided((rows, cols), (pitch, 1))
    view.copy_(t2d)
    return view


@pytest.mark.parametrize("which", ["lda", "ldb"])
def test_int8_row_pitch_beyond_32_bit_lane_offsets(which):
    M, N, K, shift = 300, 48, 256, 6
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=9103)
    want = oracle.gemm_i8(A, B, bias, shift, 0)
    Ad = strided(dev(A), (1 << 24) + 16) if which == "lda" else dev(A)   # 256 rows of A span 4 GiB
    Bd = strided(dev(B), (1 << 26) + 16) if which == "ldb" else dev(B)   # 64 rows of B span 4 GiB (256 rows: 17 GB)
    C = torch.full((M, N), 91, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8(Ad, Bd, dev(bias), C, shift, 0)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C), want)
    C32 = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    ops.ac_gemm_i8_acc32(Ad, Bd, dev(bias), C32)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C32).astype(np.int64), oracle.gemm_i8(A, B, bias, 0, 0, return_acc=True)[1])
    # a K split needs the direct-to-LDS kernels, which these operands do not qualify for
    ws = torch.empty(ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, 64, 2), dtype=torch.uint8, device="cuda")
    with pytest.raises(ops.AcError) as err:
        ops.ac_gemm_i8_planned(Ad, Bd, dev(bias), C, shift, 0, 64, 2, workspace=ws)
    assert err.value.status == ops.AC_ERR_PLAN


def test_bf16_row_pitch_beyond_32_bit_lane_offsets():
    M, N, K = 300, 48, 64
    A, B = inputs.gemm_bf16_inputs(M, N, K, seed=9104)
    want = oracle.gemm_bf16(A, B)
    Ad = strided(dev(A), (1 << 23) + 8)   # 16 MiB rows: 256 of them span 4 GiB
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ops.ac_gemm_bf16(Ad, dev(B), C, 1.0, 0.0)
    torch.cuda.synchronize()
    assert rel_fro(host(C), want) <= 1e-3
