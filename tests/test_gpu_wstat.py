"""GPU parity of the weight-stationary int8 kernel (tile codes 320 / 160) against the CPU oracle, bit for bit.

Reached through the planned entry points, so that every shape here runs on that kernel whatever the library's own
choice would be: row tiles that stream one after another through a workgroup, ragged M / N / K, partial column
blocks, every output-stage variant, and the convolution gather with its incremental pixel bookkeeping.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu

TILES = (320, 160)


def gemm_check(A, B, bias, shift, act, tile):
    M, N = A.shape[0], B.shape[1]
    C = torch.full((M, N), 77, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8_planned(dev(A), dev(B), dev(bias), C, shift, act, tile, 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C), oracle.gemm_i8(A, B, bias, shift, act))


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("M,N,K", [
    (1, 16, 16), (64, 16, 128), (257, 64, 144), (1000, 64, 576), (3136, 64, 576), (300, 128, 64), (777, 48, 208),
    (600, 112, 400), (5000, 64, 1536), (12544, 64, 256), (3136, 256, 64), (333, 320, 96),
    (100000, 64, 320),   # 391 / 782 row tiles: every workgroup streams several tiles
    (70001, 128, 192),   # two column blocks, ragged last row tile
])
def test_gemm_shapes(M, N, K, tile):
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + N + K)
    gemm_check(A, B, bias, 9, ops.AC_ACT_RELU, tile)
    if M <= 5000:
        gemm_check(A, B, None, 6, ops.AC_ACT_NONE, tile)


def test_deepest_resident_k():
    A, B, bias = inputs.gemm_i8_inputs(700, 80, 2048, seed=5)
    gemm_check(A, B, bias, 11, 1, 160)
    with pytest.raises(ops.AcError) as e:
        gemm_check(A, B, bias, 11, 1, 320)  # 16 K tiles do not fit beside the 256-row ring
    assert e.value.status == ops.AC_ERR_PLAN


@pytest.mark.parametrize("shift", [0, 1, 5, 8, 16, 23, 24, 31])
@pytest.mark.parametrize("act", [0, 1])
def test_shifts_and_activation(shift, act):
    A, B, bias = inputs.gemm_i8_inputs(300, 64, 160, seed=shift, bias_bits=30 if shift > 16 else 15)
    gemm_check(A, B, bias, shift, act, 160)


def test_small_magnitudes_and_ties():
    for shift in (1, 2, 3, 4):
        A, B, bias = inputs.gemm_i8_inputs(300, 96, 64, seed=shift, lo=-4, hi=4, bias_bits=4)
        gemm_check(A, B, bias, shift, 0, 160)
        gemm_check(A, B, bias, shift, 1, 320)
    # acc = K + bias sweeps every multiple of half a step
    M, N, K, shift = 64, 256, 16, 4
    A = np.ones((M, K), np.int8)
    B = np.ones((K, N), np.int8)
    bias = ((np.arange(N, dtype=np.int64) - 128) * 8 - K).astype(np.int32)
    gemm_check(A, B, bias, shift, 0, 160)


def test_extreme_accumulators():
    # sums near the ends of int32: the rounding add must not wrap
    M, N, K = 64, 64, 16
    A = np.zeros((M, K), np.int8)
    B = np.zeros((K, N), np.int8)
    edge = np.array([2**31 - 1, 2**31 - 2, -(2**31), -(2**31) + 1, 2**30, 2**30 - 1, -(2**30), -(2**30) - 1], dtype=np.int64)
    bias = np.resize(edge, N).astype(np.int32)
    for shift in (1, 8, 23, 24, 31):
        gemm_check(A, B, bias, shift, 0, 160)


def test_plan_errors():
    A, B, bias = inputs.gemm_i8_inputs(128, 64, 128, seed=1)
    full = np.zeros((128, 64), np.int32)
    C = torch.empty((128, 64), dtype=torch.int8, device="cuda")
    with pytest.raises(ops.AcError) as e:
        ops.ac_gemm_i8_planned(dev(A), dev(B), dev(full), C, 8, 1, 320, 1)  # a bias matrix
    assert e.value.status == ops.AC_ERR_PLAN
    with pytest.raises(ops.AcError) as e:
        ops.ac_gemm_i8_planned(dev(A), dev(B), dev(bias), C, 8, 1, 320, 2)  # no K split on this kernel
    assert e.value.status == ops.AC_ERR_PLAN
    A2, B2, bias2 = inputs.gemm_i8_inputs(128, 60, 128, seed=1)  # N not a multiple of 16
    C2 = torch.empty((128, 60), dtype=torch.int8, device="cuda")
    with pytest.raises(ops.AcError) as e:
        ops.ac_gemm_i8_planned(dev(A2), dev(B2), dev(bias2), C2, 8, 1, 160, 1)
    assert e.value.status == ops.AC_ERR_PLAN


def conv_check(x, w, bias, stride, pad, shift, act, tile):
    Nb, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    OH = (H + 2 * pad - KH) // stride + 1
    OW = (W + 2 * pad - KW) // stride + 1
    out = torch.full((Nb, OH, OW, Cout), 99, dtype=torch.int8, device="cuda")
    ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, stride, pad, shift, act, plan=(tile, 1))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(out), oracle.conv2d_i8(x, w, bias, stride, pad, shift, act))


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("Nb,H,W,Cin,Cout,KH,KW,stride,pad", [
    (1, 5, 5, 16, 16, 3, 3, 1, 1),
    (2, 9, 7, 16, 32, 3, 3, 2, 1),
    (3, 12, 12, 32, 48, 3, 3, 1, 0),
    (2, 14, 14, 64, 64, 1, 1, 1, 0),
    (1, 6, 6, 16, 16, 5, 5, 1, 2),
    (1, 3, 3, 16, 16, 5, 5, 1, 1),
    (4, 30, 30, 48, 80, 3, 3, 1, 1),
    (2, 17, 23, 16, 272, 3, 3, 3, 2),
    (8, 56, 56, 64, 64, 3, 3, 1, 1),     # the stride-1 workload
    (8, 28, 28, 128, 256, 3, 3, 2, 1),   # the stride-2 workload
    (9, 61, 67, 16, 16, 3, 3, 1, 1),     # 288 row tiles of 128: some workgroups take two, odd image sizes
    (20, 61, 67, 16, 32, 3, 3, 1, 1),    # 320 row tiles of 256
    (70, 31, 29, 32, 16, 2, 3, 2, 0),    # stride 2, KH != KW, many tiles per workgroup for 128-row tiles
])
def test_conv_shapes(Nb, H, W, Cin, Cout, KH, KW, stride, pad, tile):
    x, w, bias = inputs.conv_i8_inputs(Nb, H, W, Cin, Cout, KH, KW, seed=H * W + Cin)
    conv_check(x, w, bias, stride, pad, 8, 1, tile)
    if Nb * H * W <= 4000:
        conv_check(x, w, None, stride, pad, 5, 0, tile)


def test_conv_plan_errors():
    x, w, bias = inputs.conv_i8_inputs(1, 8, 8, 3, 8, 3, 3, seed=1)  # Cin not a multiple of 16
    out = torch.empty((1, 8, 8, 8), dtype=torch.int8, device="cuda")
    with pytest.raises(ops.AcError) as e:
        ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, 1, 1, 8, 1, plan=(160, 1))
    assert e.value.status == ops.AC_ERR_PLAN
    x, w, bias = inputs.conv_i8_inputs(1, 8, 8, 16, 16, 3, 3, seed=1)
    out = torch.empty((1, 8, 8, 16), dtype=torch.int8, device="cuda")
    with pytest.raises(ops.AcError) as e:
        ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, 1, 1, 8, 1, plan=(77, 1))  # unknown tile
    assert e.value.status == ops.AC_ERR_PLAN
    ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, 1, 1, 8, 1, plan=(64, 1))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(out), oracle.conv2d_i8(x, w, bias, 1, 1, 8, 1))


# ---- the convolution patch kernel (tile codes 321 / 161): weights and the image patch of a unit both in LDS ----

PATCH_TILES = (321, 161)


@pytest.mark.parametrize("tile", PATCH_TILES)
@pytest.mark.parametrize("Nb,H,W,Cin,Cout,KH,KW,stride,pad", [
    (1, 5, 5, 32, 16, 3, 3, 1, 1),
    (2, 9, 7, 32, 32, 3, 3, 2, 1),       # stride 2, odd image: two column planes of unequal width
    (3, 12, 12, 32, 48, 3, 3, 1, 0),     # no padding
    (2, 14, 14, 64, 64, 1, 1, 1, 0),     # 1x1
    (1, 6, 6, 32, 16, 5, 5, 1, 2),       # 5x5
    (1, 3, 3, 32, 16, 5, 5, 1, 1),       # kernel larger than the image
    (4, 30, 30, 96, 80, 3, 3, 1, 1),     # Cin not a power of two, a partial second column block
    (2, 17, 23, 32, 272, 3, 3, 3, 2),    # stride 3, pad 2, five column blocks
    (8, 56, 56, 64, 64, 3, 3, 1, 1),     # the stride-1 workload
    (9, 61, 67, 32, 16, 3, 3, 1, 1),     # odd row length: units start and end mid-row
    (70, 31, 29, 32, 16, 2, 3, 2, 0),    # stride 2, KH != KW
    (3, 20, 300, 32, 32, 3, 3, 1, 1),    # rows longer than a unit
    (40, 56, 56, 64, 64, 3, 3, 1, 1),    # 520 / 1000 units: every workgroup streams several
])
def test_patch_kernel_shapes(Nb, H, W, Cin, Cout, KH, KW, stride, pad, tile):
    x, w, bias = inputs.conv_i8_inputs(Nb, H, W, Cin, Cout, KH, KW, seed=H * W + Cin)
    conv_check(x, w, bias, stride, pad, 8, 1, tile)
    if Nb * H * W <= 4000:
        conv_check(x, w, None, stride, pad, 5, 0, tile)


def test_patch_kernel_small_magnitudes():
    x, w, bias = inputs.conv_i8_inputs(2, 9, 9, 32, 32, 3, 3, seed=1, lo=-3, hi=3, bias_bits=4)
    for shift in (0, 1, 2, 3):
        conv_check(x, w, bias, 1, 1, shift, 0, 161)


def test_patch_kernel_plan_errors():
    # the stride-2 workload: its patch (a whole 28 x 28 x 128 image) and 72 KB of weights do not fit in LDS together
    x, w, bias = inputs.conv_i8_inputs(2, 28, 28, 128, 256, 3, 3, seed=1)
    out = torch.empty((2, 14, 14, 256), dtype=torch.int8, device="cuda")
    for tile in PATCH_TILES:
        with pytest.raises(ops.AcError) as e:
            ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, 2, 1, 9, 1, plan=(tile, 1))
        assert e.value.status == ops.AC_ERR_PLAN
    x, w, bias = inputs.conv_i8_inputs(1, 8, 8, 16, 16, 3, 3, seed=1)  # Cin = 16: a K-step would straddle two taps
    out = torch.empty((1, 8, 8, 16), dtype=torch.int8, device="cuda")
    with pytest.raises(ops.AcError) as e:
        ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, 1, 1, 8, 1, plan=(161, 1))
    assert e.value.status == ops.AC_ERR_PLAN
    A, B, b = inputs.gemm_i8_inputs(128, 64, 128, seed=1)  # not a GEMM kernel
    C = torch.empty((128, 64), dtype=torch.int8, device="cuda")
    with pytest.raises(ops.AcError) as e:
        ops.ac_gemm_i8_planned(dev(A), dev(B), dev(b), C, 8, 1, 321, 1)
    assert e.value.status == ops.AC_ERR_PLAN


# ---- the library's own choice: shapes that ac_gemm_i8 / ac_conv2d_i8 hand to these kernels by themselves ----

@pytest.mark.parametrize("M,N,K", [(60000, 32, 16), (49153, 80, 272), (50000, 128, 256),
                                   (2048, 4096, 512), (4096, 4096, 128), (3000, 1100, 200), (1024, 3072, 512)])
def test_gemm_auto_choice(M, N, K):
    """Shapes whose lowest time estimate is the weight-stationary kernel's: long and narrow ones, and wide ones
    with a short K (every 64-column block then has its own workgroups, up to several rounds of them)."""
    assert ops.ac_gemm_i8_auto_plan(M, N, K, True) == (320, 1)
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + N + K)
    C = torch.full((M, N), 77, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8(dev(A), dev(B), dev(bias), C, 9, ops.AC_ACT_RELU)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C), oracle.gemm_i8(A, B, bias, 9, 1))
    # a bias matrix is not something the weight-stationary kernel takes: the same call falls back to the tiled kernels
    if M <= 50000:
        _, _, full = inputs.gemm_i8_inputs(M, N, K, seed=M + N + K + 1, bias_matrix=True)
        ops.ac_gemm_i8(dev(A), dev(B), dev(full), C, 9, ops.AC_ACT_NONE)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(C), oracle.gemm_i8(A, B, full, 9, 0))


def test_conv_auto_choice():
    # 24 images of 56 x 56 x 64 -> 64: 312 units of 256 output pixels, which the library runs on the patch kernel
    x, w, bias = inputs.conv_i8_inputs(24, 56, 56, 64, 64, 3, 3, seed=77)
    out = torch.full((24, 56, 56, 64), 99, dtype=torch.int8, device="cuda")
    ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, 1, 1, 9, ops.AC_ACT_RELU)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(out), oracle.conv2d_i8(x, w, bias, 1, 1, 9, 1))
