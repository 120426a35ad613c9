"""Pins for the int8 convolution oracle (direct definition; Section 4.4.2 workload)."""
import numpy as np
import pytest

import oracle
from conftest import read_golden_table
from paper_2505_18574_amd import inputs


def brute_conv(x, w, bias, stride, pad, shift, relu):
    Nb, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    OH = (H + 2 * pad - KH) // stride + 1
    OW = (W + 2 * pad - KW) // stride + 1
    xp = np.zeros((Nb, H + 2 * pad, W + 2 * pad, Cin), dtype=np.int64)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    out = np.zeros((Nb, OH, OW, Cout), dtype=np.int8)
    for n in range(Nb):
        for oh in range(OH):
            for ow in range(OW):
                patch = xp[n, oh * stride:oh * stride + KH, ow * stride:ow * stride + KW, :]
                for co in range(Cout):
                    s = int((patch * w[:, :, :, co].astype(np.int64)).sum())
                    if bias is not None:
                        s += int(bias[co])
                    out[n, oh, ow, co] = oracle.requantise(s, shift, relu)
    return out


@pytest.mark.parametrize("H,W,KH,KW,stride,pad", [(5, 5, 3, 3, 1, 1), (5, 4, 3, 3, 2, 1), (4, 5, 1, 1, 1, 0),
                                                  (5, 5, 3, 2, 1, 0), (4, 4, 3, 3, 2, 0), (3, 3, 3, 3, 1, 2)])
def test_brute_force_tiny(H, W, KH, KW, stride, pad):
    x, w, bias = inputs.conv_i8_inputs(2, H, W, 3, 4, KH, KW, seed=H * 10 + W)
    for shift, relu in ((0, 0), (6, 1)):
        got = oracle.conv2d_i8(x, w, bias, stride, pad, shift, relu)
        np.testing.assert_array_equal(got, brute_conv(x, w, bias, stride, pad, shift, relu))


@pytest.mark.parametrize("Nb,H,W,Cin,Cout,KH,KW,stride,pad", [
    (2, 9, 9, 16, 8, 3, 3, 1, 1), (1, 10, 8, 5, 7, 3, 3, 2, 1), (3, 6, 6, 4, 4, 1, 1, 1, 0), (1, 7, 7, 8, 3, 5, 5, 2, 2)])
def test_conv_equals_im2col_gemm(Nb, H, W, Cin, Cout, KH, KW, stride, pad):
    x, w, bias = inputs.conv_i8_inputs(Nb, H, W, Cin, Cout, KH, KW, seed=21)
    direct = oracle.conv2d_i8(x, w, bias, stride, pad, 7, 1)
    col = oracle.im2col_i8(x, KH, KW, stride, pad)
    via_gemm = oracle.gemm_i8(col, w.reshape(KH * KW * Cin, Cout), bias, 7, 1)
    np.testing.assert_array_equal(direct.reshape(-1, Cout), via_gemm)


def test_1x1_is_a_gemm_over_pixels():
    x, w, bias = inputs.conv_i8_inputs(2, 6, 5, 12, 9, 1, 1, seed=22)
    got = oracle.conv2d_i8(x, w, bias, 1, 0, 5, 0)
    want = oracle.gemm_i8(x.reshape(-1, 12), w.reshape(12, 9), bias, 5, 0)
    np.testing.assert_array_equal(got.reshape(-1, 9), want)


def test_delta_kernel_is_identity():
    x, _, _ = inputs.conv_i8_inputs(2, 7, 6, 5, 5, 3, 3, seed=23)
    w = np.zeros((3, 3, 5, 5), dtype=np.int8)
    w[1, 1] = np.eye(5, dtype=np.int8)
    np.testing.assert_array_equal(oracle.conv2d_i8(x, w, None, 1, 1, 0, 0), x)
    # a delta at tap (0, 0) shifts the image down-right by one pixel (zero fill)
    w[:] = 0
    w[0, 0] = np.eye(5, dtype=np.int8)
    got = oracle.conv2d_i8(x, w, None, 1, 1, 0, 0)
    want = np.zeros_like(x)
    want[:, 1:, 1:, :] = x[:, :-1, :-1, :]
    np.testing.assert_array_equal(got, want)


def test_all_ones_counts_taps():
    for H, W, KH, KW, stride, pad, oh, ow, taps in read_golden_table("conv_ones_taps.txt"):
        Cin = 3
        x = np.ones((1, H, W, Cin), dtype=np.int8)
        w = np.ones((KH, KW, Cin, 2), dtype=np.int8)
        got = oracle.conv2d_i8(x, w, None, stride, pad, 0, 0)
        assert got[0, oh, ow, 0] == taps * Cin, (H, W, KH, KW, stride, pad, oh, ow)
        assert got[0, oh, ow, 1] == taps * Cin


def test_output_shape_floor_formula():
    x, w, bias = inputs.conv_i8_inputs(1, 28, 28, 4, 4, 3, 3, seed=24)
    assert oracle.conv2d_i8(x, w, bias, 2, 1, 9, 1).shape == (1, 14, 14, 4)
    x, w, bias = inputs.conv_i8_inputs(1, 8, 7, 4, 4, 3, 3, seed=24)
    assert oracle.conv2d_i8(x, w, bias, 2, 0, 9, 1).shape == (1, 3, 3, 4)
    for case in inputs.CONV_I8:
        assert (case.OH, case.OW) == ((56, 56) if case.stride == 1 else (14, 14))
    assert inputs.CONV_I8[0].gemm_mnk == (25088, 64, 576) and inputs.CONV_I8[1].gemm_mnk == (1568, 256, 1152)
