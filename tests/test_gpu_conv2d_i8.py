"""GPU parity: ac_conv2d_i8 against the direct-definition oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu


def check(x, w, bias, stride, pad, shift, act):
    Nb, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    OH = (H + 2 * pad - KH) // stride + 1
    OW = (W + 2 * pad - KW) // stride + 1
    want = oracle.conv2d_i8(x, w, bias, stride, pad, shift, act)
    for with_ws in (False, True):  # with a workspace the library may split the K range
        out = torch.full((Nb, OH, OW, Cout), 99, dtype=torch.int8, device="cuda")
        ws = None
        if with_ws:
            nbytes = ops.ac_gemm_i8_workspace_bytes(Nb * OH * OW, Cout, KH * KW * Cin)
            if not nbytes:
                continue
            ws = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device="cuda")  # contents on entry are unspecified
        ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, stride, pad, shift, act, workspace=ws)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(out), want)


@pytest.mark.parametrize("case", inputs.CONV_I8, ids=lambda c: c.name)
def test_workload_configs(case):
    x, w, bias = inputs.conv_i8_case_inputs(case)
    check(x, w, bias, case.stride, case.pad, case.shift, case.act)


@pytest.mark.parametrize("Nb,H,W,Cin,Cout,KH,KW,stride,pad", [
    (1, 5, 5, 16, 16, 3, 3, 1, 1),      # one tile
    (2, 9, 7, 16, 32, 3, 3, 2, 1),      # stride 2, odd image
    (3, 12, 12, 32, 48, 3, 3, 1, 0),    # no padding
    (1, 8, 8, 3, 8, 3, 3, 1, 1),        # Cin not a multiple of 16: element-wise gather path
    (2, 10, 6, 5, 7, 3, 2, 2, 1),       # nothing aligned, KH != KW
    (2, 14, 14, 64, 64, 1, 1, 1, 0),    # 1x1: a plain GEMM over pixels
    (1, 6, 6, 16, 16, 5, 5, 1, 2),      # 5x5
    (1, 4, 4, 16, 16, 4, 4, 1, 0),      # kernel as large as the image: one output pixel
    (1, 3, 3, 16, 16, 5, 5, 1, 1),      # kernel larger than the image, fits only through padding
    (4, 30, 30, 48, 80, 3, 3, 1, 1),    # many tiles, ragged in M and N
    (2, 17, 23, 16, 272, 3, 3, 3, 2),   # stride 3, pad 2
    (1, 14, 14, 256, 64, 3, 3, 1, 1),   # few tiles, deep K
    (2, 7, 7, 512, 128, 3, 3, 1, 1),
    (1, 7, 7, 1024, 64, 3, 3, 1, 1),    # one tile, 72 K tiles: split-K when a workspace is given
    (1, 9, 9, 16, 16, 4, 8, 1, 3),      # 32 kernel taps: the most the tap bit mask of the tiled gather holds
    (1, 10, 10, 16, 32, 6, 6, 1, 2),    # 36 taps: beyond the mask, the element-wise gather takes it
    (1, 12, 12, 16, 16, 7, 7, 2, 3),    # 7x7 stride 2
    (2, 5, 7, 48, 16, 3, 3, 1, 3),      # padding wider than the kernel: border outputs see no input at all
    (1, 6, 20, 32, 16, 1, 5, 1, 2),     # one kernel row
    (2, 8, 8, 16, 16, 2, 2, 2, 0),      # non-overlapping windows
    (3, 11, 13, 80, 96, 3, 3, 2, 1),    # Cin not a power of two, odd image, stride 2
    (4, 28, 28, 256, 64, 1, 1, 1, 0),   # 1x1 over every pixel: handed to the GEMM kernels
    (2, 9, 9, 24, 40, 1, 1, 1, 0),      # ... with channel counts the direct-to-LDS path does not take
    (2, 9, 9, 32, 32, 1, 1, 2, 0),      # 1x1 with a stride: still a gather
    (1, 8, 8, 16, 16, 1, 1, 1, 1),      # 1x1 with padding: border outputs are the bias alone
    (16, 56, 56, 64, 256, 1, 1, 1, 0),  # 1x1 with a short K and many pixels: the weight-stationary GEMM kernel
])
def test_shapes(Nb, H, W, Cin, Cout, KH, KW, stride, pad):
    x, w, bias = inputs.conv_i8_inputs(Nb, H, W, Cin, Cout, KH, KW, seed=H * W + Cin)
    check(x, w, bias, stride, pad, 8, 1)
    check(x, w, None, stride, pad, 5, 0)


@pytest.mark.parametrize("case", inputs.CONV_I8, ids=lambda c: c.name)
def test_batch_256_sampled_images(case):
    """The workload convolutions at batch 256, as the benchmark's scale-up lines launch them (the library then
    picks its large-problem kernels): images are independent, so whole output images are checked against the
    oracle run on those images alone, and the last image guards the end of the buffers."""
    Nb = 256
    x, w, bias = inputs.conv_i8_inputs(Nb, case.H, case.W, case.Cin, case.Cout, case.KH, case.KW, seed=case.seed + 7)
    out = torch.full((Nb, case.OH, case.OW, case.Cout), 99, dtype=torch.int8, device="cuda")
    ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, case.stride, case.pad, case.shift, case.act)
    torch.cuda.synchronize()
    got = host(out)
    picks = [0, 1, 100, 191, 254, 255]
    want = oracle.conv2d_i8(np.ascontiguousarray(x[picks]), w, bias, case.stride, case.pad, case.shift, case.act)
    np.testing.assert_array_equal(got[picks], want)
    # images the oracle did not see: an image that equals a checked one must produce that one's output
    x2 = x.copy()
    x2[7] = x[100]
    x2[200] = x[0]
    ops.ac_conv2d_i8(dev(x2), dev(w), dev(bias), out, case.stride, case.pad, case.shift, case.act)
    torch.cuda.synchronize()
    got2 = host(out)
    np.testing.assert_array_equal(got2[7], want[2])
    np.testing.assert_array_equal(got2[200], want[0])
    np.testing.assert_array_equal(got2[picks], want)


def test_small_magnitudes():
    x, w, bias = inputs.conv_i8_inputs(2, 9, 9, 16, 32, 3, 3, seed=1, lo=-3, hi=3, bias_bits=4)
    for shift in (0, 1, 2, 3):
        check(x, w, bias, 1, 1, shift, 0)


def test_empty_and_errors():
    L = ops.lib()
    a = torch.zeros(4096, dtype=torch.int8, device="cuda").data_ptr()
    # batch of zero images: accepted, no launch
    assert L.ac_conv2d_i8(a, a + 1024, None, a + 2048, 0, 5, 5, 16, 16, 3, 3, 1, 1, 8, 1, None, 0, None) == 0
    assert L.ac_conv2d_i8(a, a + 1024, None, a + 2048, 1, 5, 5, 16, 16, 9, 3, 1, 1, 8, 1, None, 0, None) == ops.AC_ERR_SHAPE
    assert L.ac_conv2d_i8(a, a + 1024, None, a + 2048, 1, 5, 5, 16, 16, 3, 3, 0, 1, 8, 1, None, 0, None) == ops.AC_ERR_SHAPE
    assert L.ac_conv2d_i8(a, a + 1024, None, a, 1, 5, 5, 16, 16, 3, 3, 1, 1, 8, 1, None, 0, None) == ops.AC_ERR_ALIAS
    assert L.ac_conv2d_i8(None, a + 1024, None, a + 2048, 1, 5, 5, 16, 16, 3, 3, 1, 1, 8, 1, None, 0, None) == ops.AC_ERR_NULL
    assert L.ac_conv2d_i8(a, a + 1024, None, a + 2048, 1, 5, 5, 16, 16, 3, 3, 1, 1, 40, 1, None, 0, None) == ops.AC_ERR_SHIFT


@pytest.mark.parametrize("plan", [None, (321, 1), (161, 1), (64, 1), (32, 1)])
def test_sums_around_the_clamp_bounds(plan):
    """Zero image, so every sum is its bias: the sums next to the clamp bounds of the rounding shift and the ends of
    int32, through the library's choice, the patch kernel, the tiled gather and the one-wave-per-tile kernel."""
    Nb, H, W, Cin, Cout = 2, 16, 16, 64, 128
    x = np.zeros((Nb, H, W, Cin), np.int8)
    w = np.ones((3, 3, Cin, Cout), np.int8)
    for shift in (1, 9, 17, 18, 23):
        half = 1 << (shift - 1)
        centres = [(127 << shift) + half - 1, 127 << shift, -(128 << shift), -(128 << shift) - half, 0, half, -half, 2**31 - 1, -(2**31)]
        vals = np.array([c + d for c in centres for d in (-2, -1, 0, 1, 2)], dtype=np.int64)
        bias = np.resize(np.clip(vals, -(2**31), 2**31 - 1), Cout).astype(np.int32)
        for act in (0, 1):
            want = oracle.conv2d_i8(x, w, bias, 1, 1, shift, act)
            out = torch.full((Nb, H, W, Cout), 99, dtype=torch.int8, device="cuda")
            ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, 1, 1, shift, act, plan=plan)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(host(out), want)
