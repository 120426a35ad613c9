"""GPU parity of the one-wave-per-tile int8 kernel (tile code 32) against the CPU oracle, bit for bit.

Reached through the planned entry point, so that every shape here runs on that kernel whatever the library's own
choice would be, and through ac_gemm_i8 on the shapes for which the library picks it: K of one to many stages of the
private LDS ring (64- and 128-byte stages; every ring depth and workgroup size the launcher picks from), ragged M
and N, workgroups whose last waves have no tile, every output-stage variant.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu


def planned_check(A, B, bias, shift, act):
    M, N = A.shape[0], B.shape[1]
    C = torch.full((M, N), 77, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8_planned(dev(A), dev(B), dev(bias), C, shift, act, 32, 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C), oracle.gemm_i8(A, B, bias, shift, act))


# K from one stage to well past the ring (3 or 6 stages), odd and even stage counts, both stage widths
@pytest.mark.parametrize("K", [64, 128, 192, 256, 320, 384, 448, 512, 576, 640, 704, 768, 1024, 1088, 2048, 4160])
def test_k_depths(K):
    A, B, bias = inputs.gemm_i8_inputs(100, 80, K, seed=K)
    planned_check(A, B, bias, 10, ops.AC_ACT_RELU)


@pytest.mark.parametrize("M,N,K", [
    (1, 16, 64), (31, 16, 128), (32, 32, 64), (33, 48, 192), (65, 80, 320), (256, 256, 256), (257, 272, 448),
    (3136, 64, 576), (3136, 256, 64), (784, 128, 1152), (49, 2048, 512), (1000, 16, 640),
    (5000, 1008, 128),   # 4 945 tiles: far more workgroups than compute units
    (1000, 272, 384), (3136, 256, 256),   # more than 256 tiles, 128-byte stages: two waves per workgroup
    (1056, 288, 256),    # 297 tiles: the last workgroup's second wave has none
    (128, 1024, 3072), (196, 1024, 2304),   # few tiles, deep K: one wave per workgroup
])
def test_shapes(M, N, K):
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + N + K)
    planned_check(A, B, bias, 9, ops.AC_ACT_RELU)
    planned_check(A, B, None, 6, ops.AC_ACT_NONE)


@pytest.mark.parametrize("shift", [0, 1, 5, 8, 16, 23, 24, 31])
@pytest.mark.parametrize("act", [0, 1])
def test_shifts_and_activation(shift, act):
    A, B, bias = inputs.gemm_i8_inputs(100, 96, 192, seed=shift, bias_bits=30 if shift > 16 else 15)
    planned_check(A, B, bias, shift, act)


def test_bias_matrix_ties_and_extreme_accumulators():
    A, B, bias = inputs.gemm_i8_inputs(150, 144, 128, seed=5, bias_matrix=True)
    planned_check(A, B, bias, 8, 1)
    for shift in (1, 2, 3, 4):  # small sums: rounding, not saturation, decides
        A, B, bias = inputs.gemm_i8_inputs(100, 96, 64, seed=shift, lo=-4, hi=4, bias_bits=4)
        planned_check(A, B, bias, shift, 0)
    # acc = K + bias sweeps every multiple of half a step
    M, N, K, shift = 64, 256, 64, 4
    A = np.ones((M, K), np.int8)
    B = np.ones((K, N), np.int8)
    bias = ((np.arange(N, dtype=np.int64) - 128) * 8 - K).astype(np.int32)
    planned_check(A, B, bias, shift, 0)
    # sums at the ends of int32: the rounding add must not wrap
    A = np.zeros((M, K), np.int8)
    edge = np.array([2**31 - 1, 2**31 - 2, -(2**31), -(2**31) + 1, 2**30, 2**30 - 1, -(2**30), -(2**30) - 1], dtype=np.int64)
    bias = np.resize(edge, N).astype(np.int32)
    for shift in (1, 8, 23, 24, 31):
        planned_check(A, B, bias, shift, 0)


def test_strided_operands_and_guard_bands():
    """Row pitches beyond the row length, and nothing written outside the M x N window of C."""
    M, N, K = 70, 48, 192
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=11)
    Ap = torch.zeros((M, K + 64), dtype=torch.int8, device="cuda")
    Bp = torch.zeros((K, N + 32), dtype=torch.int8, device="cuda")
    Ap[:, :K] = dev(A)
    Bp[:, :N] = dev(B)
    Cp = torch.full((M + 2, N + 16), 55, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8_planned(Ap[:, :K], Bp[:, :N], dev(bias), Cp[1:M + 1, :N], 9, 1, 32, 1)
    torch.cuda.synchronize()
    got = host(Cp)
    np.testing.assert_array_equal(got[1:M + 1, :N], oracle.gemm_i8(A, B, bias, 9, 1))
    assert (got[0] == 55).all() and (got[M + 1] == 55).all() and (got[:, N:] == 55).all()


def test_refusals_and_fallbacks():
    A, B, bias = inputs.gemm_i8_inputs(64, 64, 96, seed=3)
    C = torch.zeros((64, 64), dtype=torch.int8, device="cuda")
    with pytest.raises(ops.AcError) as e:  # K not in whole 64-byte stages
        ops.ac_gemm_i8_planned(dev(A), dev(B), dev(bias), C, 8, 0, 32, 1)
    assert e.value.status == ops.AC_ERR_PLAN
    A, B, bias = inputs.gemm_i8_inputs(64, 64, 128, seed=3)
    with pytest.raises(ops.AcError) as e:  # more slices than K tiles of 64 bytes
        ops.ac_gemm_i8_planned(dev(A), dev(B), dev(bias), C, 8, 0, 32, 3)
    assert e.value.status == ops.AC_ERR_PLAN
    with pytest.raises(ops.AcError) as e:  # operands the direct-to-LDS kernels do not take (N = 60)
        ops.ac_gemm_i8_planned(dev(A), dev(B[:, :60].copy()), dev(bias[:60].copy()), C[:, :60].contiguous(), 8, 0, 32, 1)
    assert e.value.status == ops.AC_ERR_PLAN
    # ac_gemm_i8 plans tile 32 for this size; with an unaligned A it must still run (on the generic kernel) and agree
    assert ops.ac_gemm_i8_auto_plan(64, 64, 128) == (32, 1)
    Ap = torch.zeros((64, 129), dtype=torch.int8, device="cuda")
    Ap[:, :128] = dev(A)
    ops.ac_gemm_i8(Ap[:, :128], dev(B), dev(bias), C, 8, 0)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C), oracle.gemm_i8(A, B, bias, 8, 0))


@pytest.mark.parametrize("M,N,K,splits", [
    (49, 2048, 4608, 8), (196, 1024, 2304, 4), (100, 80, 4160, 5), (33, 48, 192, 3), (1, 16, 128, 2), (300, 272, 1088, 16),
    (64, 64, 8192, 128),   # one K tile per slice
    (130, 80, 8384, 7),    # 131 K tiles in slices of 19: the last slice is shorter
])
def test_k_slices(M, N, K, splits):
    """A cut K range: every (tile, slice) is a wave of its own, the slices' int32 sums go through the workspace."""
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + N + K)
    need = ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, 32, splits)
    assert need > 0 and need % (M * N * 4) == 0
    ws = torch.full((need,), 0xA5, dtype=torch.uint8, device="cuda")  # contents on entry are unspecified
    for bias_, shift, act in ((bias, 12, 1), (None, 9, 0)):
        C = torch.full((M, N), 77, dtype=torch.int8, device="cuda")
        ops.ac_gemm_i8_planned(dev(A), dev(B), dev(bias_), C, shift, act, 32, splits, workspace=ws)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(C), oracle.gemm_i8(A, B, bias_, shift, act))
    with pytest.raises(ops.AcError) as e:  # a cut K range needs the workspace
        ops.ac_gemm_i8_planned(dev(A), dev(B), dev(bias), C, 12, 1, 32, splits)
    assert e.value.status == ops.AC_ERR_WORKSPACE


def conv_planned_check(x, w, bias, stride, pad, shift, act):
    Nb, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    OH, OW = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    out = torch.full((Nb, OH, OW, Cout), 99, dtype=torch.int8, device="cuda")
    ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, stride, pad, shift, act, plan=(32, 1))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(out), oracle.conv2d_i8(x, w, bias, stride, pad, shift, act))


# the convolution gather of the same kernel: K = KH KW Cin in whole 64-byte stages (one tap per stage, several stages
# per tap, several taps per stage), borders, strides, ragged pixel and channel counts
@pytest.mark.parametrize("Nb,H,W,Cin,Cout,KH,KW,stride,pad", [
    (1, 56, 56, 64, 64, 3, 3, 1, 1),     # one 64-byte stage per tap
    (1, 28, 28, 128, 256, 3, 3, 2, 1),   # one 128-byte stage per tap, stride 2
    (2, 9, 7, 64, 32, 3, 3, 2, 1),       # odd image
    (3, 12, 12, 32, 48, 3, 3, 1, 0),     # K = 288: not in whole stages -> refused (checked below)
    (1, 6, 6, 16, 16, 2, 2, 1, 1),       # four taps per stage
    (2, 10, 10, 32, 80, 2, 2, 2, 0),     # two taps per 64-byte stage, non-overlapping windows
    (1, 14, 14, 256, 64, 3, 3, 1, 1),    # two 128-byte stages per tap
    (1, 7, 7, 192, 48, 3, 3, 1, 1),      # 1.5 stages per tap: a stage that straddles two taps
    (2, 5, 7, 64, 16, 3, 3, 1, 3),       # padding wider than the kernel
    (1, 9, 9, 16, 16, 4, 8, 1, 3),       # 32 taps
    (4, 30, 30, 64, 80, 3, 3, 1, 1),     # 3600 pixels: many tiles, ragged in M and N
    (2, 9, 9, 64, 32, 1, 1, 2, 0),       # 1 x 1 with a stride
])
def test_convolution_gather(Nb, H, W, Cin, Cout, KH, KW, stride, pad):
    x, w, bias = inputs.conv_i8_inputs(Nb, H, W, Cin, Cout, KH, KW, seed=H * W + Cin)
    if (KH * KW * Cin) % 64:
        with pytest.raises(ops.AcError) as e:
            conv_planned_check(x, w, bias, stride, pad, 8, 1)
        assert e.value.status == ops.AC_ERR_PLAN
        return
    conv_planned_check(x, w, bias, stride, pad, 8, 1)
    conv_planned_check(x, w, None, stride, pad, 5, 0)


def test_convolution_gather_with_k_slices():
    x, w, bias = inputs.conv_i8_inputs(1, 7, 7, 512, 64, 3, 3, seed=77)  # 49 pixels, K = 4608
    M, N, K = 49, 64, 4608
    want = oracle.conv2d_i8(x, w, bias, 1, 1, 11, 1)
    for splits in (4, 9):
        need = ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, 32, splits)
        ws = torch.full((need,), 0x5A, dtype=torch.uint8, device="cuda")
        out = torch.full((1, 7, 7, 64), 99, dtype=torch.int8, device="cuda")
        ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, 1, 1, 11, 1, workspace=ws, plan=(32, splits))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(out), want)


def test_library_choice_runs_it():
    """Shapes of the accelerator-sized layers (Section 4.4.1) through ac_gemm_i8 itself."""
    for M, N, K in [(256, 256, 256), (3136, 64, 576), (3136, 256, 64), (512, 512, 512), (128, 128, 128), (128, 1024, 1024),
                    (512, 768, 768), (2048, 1024, 128)]:
        assert ops.ac_gemm_i8_auto_plan(M, N, K) == (32, 1)
        A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + K)
        C = torch.full((M, N), 77, dtype=torch.int8, device="cuda")
        ops.ac_gemm_i8(dev(A), dev(B), dev(bias), C, 9, 1)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(C), oracle.gemm_i8(A, B, bias, 9, 1))
