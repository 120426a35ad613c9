"""GPU parity on seeded random shapes: every kernel family (direct-to-LDS tiles of all three sizes, split-K,
the generic fallback, the transposed-operand kernel) is reached by shapes the directed tests do not name."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host, rel_fro
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu


def random_shapes(seed, count, aligned):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        M = int(rng.integers(1, 700))
        N = int(rng.integers(1, 700))
        K = int(rng.integers(1, 1500))
        if aligned:  # multiples of 16: the direct-to-LDS path
            N, K = max(16, N // 16 * 16), max(16, K // 16 * 16)
        out.append((M, N, K))
    # a few large ones so that the 128 and 256 tiles and a split are chosen
    out += [(2100, 2064, 208), (3100, 3088, 80), (40, 48, 4096)] if aligned else [(1500, 1700, 100)]
    return out


@pytest.mark.parametrize("aligned", [True, False])
def test_int8_random_shapes(aligned):
    for idx, (M, N, K) in enumerate(random_shapes(101 if aligned else 202, 24, aligned)):
        A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=7000 + idx, bias_matrix=(idx % 5 == 0))
        shift, act = int(idx % 13), int(idx % 2)
        want = oracle.gemm_i8(A, B, bias if idx % 7 else None, shift, act)
        C = torch.full((M, N), 91, dtype=torch.int8, device="cuda")
        nbytes = ops.ac_gemm_i8_workspace_bytes(M, N, K)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda") if nbytes and idx % 2 == 0 else None
        ops.ac_gemm_i8(dev(A), dev(B), dev(bias) if idx % 7 else None, C, shift, act, workspace=ws)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(C), want, err_msg=f"shape {(M, N, K)} shift {shift} act {act}")
        # the same product with both operands transposed in memory
        Ct = torch.full((M, N), 92, dtype=torch.int8, device="cuda")
        ops.ac_gemm_i8_t(dev(np.ascontiguousarray(A.T)), dev(np.ascontiguousarray(B.T)), dev(bias) if idx % 7 else None, Ct,
                         shift, act, trans_a=True, trans_b=True)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(Ct), want, err_msg=f"transposed, shape {(M, N, K)}")


@pytest.mark.parametrize("aligned", [True, False])
def test_bf16_random_shapes(aligned):
    for idx, (M, N, K) in enumerate(random_shapes(303 if aligned else 404, 16, aligned)):
        A, B = inputs.gemm_bf16_inputs(M, N, K, seed=8000 + idx)
        alpha, beta = (1.0, 0.0) if idx % 3 else (0.75, -1.5)
        C_in = np.random.default_rng(idx).standard_normal((M, N)).astype(np.float32)
        want = oracle.gemm_bf16(A, B, alpha, beta, C_in if beta else None)
        C = dev(C_in).clone() if beta else torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        ops.ac_gemm_bf16(dev(A), dev(B), C, alpha, beta)
        torch.cuda.synchronize()
        got = host(C)
        assert rel_fro(got, want) <= 1e-3, (M, N, K)
        Aa = np.abs(inputs.bf16_bits_to_f32(A).astype(np.float64))
        Ba = np.abs(inputs.bf16_bits_to_f32(B).astype(np.float64))
        bound = 4.0 * (K + 2) * 2.0 ** -24 * (abs(alpha) * (Aa @ Ba) + abs(beta) * np.abs(C_in)) + 1e-30
        assert (np.abs(got - want) <= bound).all(), (M, N, K)


def test_conv_random_geometries():
    rng = np.random.default_rng(505)
    for idx in range(14):
        Nb, H, W = int(rng.integers(1, 4)), int(rng.integers(3, 20)), int(rng.integers(3, 20))
        KH, KW = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        stride, pad = int(rng.integers(1, 3)), int(rng.integers(0, 2))
        if idx % 2 == 0:  # fast path: channel counts in multiples of 16
            Cin, Cout = 16 * int(rng.integers(1, 5)), 16 * int(rng.integers(1, 6))
        else:
            Cin, Cout = int(rng.integers(1, 40)), int(rng.integers(1, 50))
        x, w, b = inputs.conv_i8_inputs(Nb, H, W, Cin, Cout, KH, KW, seed=9000 + idx)
        OH, OW = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
        out = torch.full((Nb, OH, OW, Cout), 17, dtype=torch.int8, device="cuda")
        ops.ac_conv2d_i8(dev(x), dev(w), dev(b), out, stride, pad, 7, idx % 2)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(out), oracle.conv2d_i8(x, w, b, stride, pad, 7, idx % 2),
                                      err_msg=f"conv {(Nb, H, W, Cin, Cout, KH, KW, stride, pad)}")


ALL_I8_TILES = (64, 128, 192, 256, 160, 320)
PATCH_TILES = (161, 321)


def test_every_plan_on_random_int8_gemms():
    """Seeded random GEMM shapes the direct-to-LDS kernels take, each through every kernel / tile code and several K
    splits by name; a plan the library refuses (AC_ERR_PLAN: K too deep for resident weights, more slices than K
    tiles) drops out, every plan it accepts must reproduce the oracle bit for bit."""
    rng = np.random.default_rng(606)
    ran = {t: 0 for t in ALL_I8_TILES}
    for idx in range(14):
        M = int(rng.integers(1, 900))
        N = 16 * int(rng.integers(1, 40))
        K = 16 * int(rng.integers(1, 120))
        A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=9200 + idx)
        shift, act = int(idx % 11), int(idx % 2)
        want = oracle.gemm_i8(A, B, bias, shift, act)
        Ad, Bd, bd = dev(A), dev(B), dev(bias)
        for tile in ALL_I8_TILES:
            for splits in (1, 2, 5):
                need = ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, tile, splits)
                ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
                C = torch.full((M, N), 91, dtype=torch.int8, device="cuda")
                try:
                    ops.ac_gemm_i8_planned(Ad, Bd, bd, C, shift, act, tile, splits, workspace=ws)
                except ops.AcError as e:
                    assert e.status == ops.AC_ERR_PLAN, (M, N, K, tile, splits)
                    continue
                torch.cuda.synchronize()
                np.testing.assert_array_equal(host(C), want, err_msg=f"shape {(M, N, K)} plan {(tile, splits)}")
                ran[tile] += 1
    assert all(n >= 10 for n in ran.values()), ran


def test_every_plan_on_random_convolutions():
    """The same for seeded random convolution geometries (channel counts in multiples of 16), with the patch kernel
    codes added."""
    rng = np.random.default_rng(707)
    ran = {t: 0 for t in ALL_I8_TILES + PATCH_TILES}
    for idx in range(16):
        Nb, H, W = int(rng.integers(1, 7)), int(rng.integers(4, 40)), int(rng.integers(4, 40))
        KH, KW = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        stride, pad = int(rng.integers(1, 4)), int(rng.integers(0, 3))
        if KH > H + 2 * pad or KW > W + 2 * pad:
            continue
        Cin, Cout = 16 * int(rng.integers(1, 7)), 16 * int(rng.integers(1, 9))
        if idx % 2 == 0:  # every other geometry is one the patch kernel can hold in LDS: 3 x 3, few channels
            KH, KW, stride, Cin = 3, 3, 1 + idx // 2 % 2, 16 * int(rng.integers(2, 5))
        x, w, b = inputs.conv_i8_inputs(Nb, H, W, Cin, Cout, KH, KW, seed=9300 + idx)
        shift, act = 6 + idx % 5, idx % 2
        want = oracle.conv2d_i8(x, w, b, stride, pad, shift, act)
        OH, OW = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
        M, K = Nb * OH * OW, KH * KW * Cin
        xd, wd, bd = dev(x), dev(w), dev(b)
        for tile in ALL_I8_TILES + PATCH_TILES:
            for splits in (1, 3):
                need = ops.ac_gemm_i8_planned_workspace_bytes(M, Cout, K, tile, splits)
                ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
                out = torch.full((Nb, OH, OW, Cout), 17, dtype=torch.int8, device="cuda")
                try:
                    ops.ac_conv2d_i8(xd, wd, bd, out, stride, pad, shift, act, workspace=ws, plan=(tile, splits))
                except ops.AcError as e:
                    assert e.status == ops.AC_ERR_PLAN, (Nb, H, W, Cin, Cout, KH, KW, stride, pad, tile, splits)
                    continue
                torch.cuda.synchronize()
                np.testing.assert_array_equal(host(out), want,
                                              err_msg=f"conv {(Nb, H, W, Cin, Cout, KH, KW, stride, pad)} plan {(tile, splits)}")
                ran[tile] += 1
    assert all(n >= 5 for n in ran.values()), ran


def test_every_plan_on_random_bf16_gemms():
    """Seeded random bf16 shapes (N and K in multiples of 8), each through every tile code and several K splits, the
    slices summed through a workspace and with atomic adds; every accepted plan within the bf16 bar of the oracle."""
    rng = np.random.default_rng(808)
    ran = 0
    for idx in range(10):
        M = int(rng.integers(1, 700))
        N = 8 * int(rng.integers(1, 70))
        K = 8 * int(rng.integers(1, 260))
        A, B = inputs.gemm_bf16_inputs(M, N, K, seed=9400 + idx)
        alpha, beta = (1.0, 0.0) if idx % 2 else (-0.5, 2.0)
        C_in = np.random.default_rng(idx).standard_normal((M, N)).astype(np.float32)
        want = oracle.gemm_bf16(A, B, alpha, beta, C_in if beta else None)
        Ad, Bd = dev(A), dev(B)
        for tile in (64, 128, 192, 256):
            for splits in (1, 2, 5):
                for with_ws in ((False,) if splits == 1 else (False, True)):
                    need = ops.ac_gemm_bf16_planned_workspace_bytes(M, N, K, tile, splits) if with_ws else 0
                    ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
                    C = dev(C_in).clone() if beta else torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
                    try:
                        ops.ac_gemm_bf16_planned(Ad, Bd, C, alpha, beta, tile, splits, workspace=ws)
                    except ops.AcError as e:
                        assert e.status == ops.AC_ERR_PLAN, (M, N, K, tile, splits)
                        continue
                    torch.cuda.synchronize()
                    assert rel_fro(host(C), want) <= 1e-3, (M, N, K, tile, splits, with_ws)
                    ran += 1
    assert ran >= 150, ran
