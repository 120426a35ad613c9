"""GPU parity: ac_gemm_i8 against the CPU oracle, bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu


def run_gpu(A, B, bias, shift, act, workspace=False):
    M, K = A.shape
    N = B.shape[1]
    C = torch.full((M, N), 77, dtype=torch.int8, device="cuda")
    ws = None
    if workspace:
        nbytes = ops.ac_gemm_i8_workspace_bytes(M, N, K)
        if nbytes:
            ws = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")  # contents on entry are unspecified
    ops.ac_gemm_i8(dev(A), dev(B), dev(bias), C, shift, act, workspace=ws)
    torch.cuda.synchronize()
    return host(C)


def check(A, B, bias, shift, act, workspace=False):
    got = run_gpu(A, B, bias, shift, act, workspace)
    want = oracle.gemm_i8(A, B, bias, shift, act)
    np.testing.assert_array_equal(got, want)


def test_config_256():
    case = inputs.GEMM_I8_256
    A, B, bias = inputs.gemm_i8_case_inputs(case)
    check(A, B, bias, case.shift, case.act)


@pytest.mark.parametrize("case", inputs.GEMM_I8_SWEEP, ids=lambda c: c.name)
@pytest.mark.parametrize("workspace", [False, True], ids=["nows", "ws"])
def test_shape_sweep(case, workspace):
    A, B, bias = inputs.gemm_i8_case_inputs(case)
    check(A, B, bias, case.shift, case.act, workspace)


# several tiles plus ragged tails in every dimension; aligned and unaligned leading dimensions;
# shapes that select each block-tile size
@pytest.mark.parametrize("M,N,K", [
    (1, 1, 1), (3, 5, 7), (64, 64, 128), (65, 63, 129), (130, 200, 100), (320, 208, 144), (257, 272, 400),
    (1792, 1792, 200), (1800, 1790, 72), (4096, 3072, 64), (4100, 3080, 48), (49, 2048, 300), (1000, 16, 1000)])
def test_ragged_shapes(M, N, K):
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + N + K)
    check(A, B, bias, 9, ops.AC_ACT_RELU)
    check(A, B, None, 7, ops.AC_ACT_NONE)


@pytest.mark.parametrize("shift", [0, 1, 5, 8, 16, 31])
@pytest.mark.parametrize("act", [0, 1])
def test_shifts_and_activation(shift, act):
    A, B, bias = inputs.gemm_i8_inputs(96, 80, 160, seed=shift, bias_bits=30 if shift > 16 else 15)
    check(A, B, bias, shift, act)


def test_small_magnitudes_and_ties():
    # inputs in [-4, 4]: sums stay small so that rounding (not saturation) decides the outputs
    for shift in (1, 2, 3, 4):
        A, B, bias = inputs.gemm_i8_inputs(128, 96, 64, seed=shift, lo=-4, hi=4, bias_bits=4)
        check(A, B, bias, shift, 0)
    # constructed ties: A = ones column, B = ones row, bias sweeps every residue -> acc = K + bias
    M, N, K, shift = 64, 256, 16, 4
    A = np.ones((M, K), np.int8)
    B = np.ones((K, N), np.int8)
    bias = ((np.arange(N, dtype=np.int64) - 128) * 8 - K).astype(np.int32)  # acc = 8 * (j - 128): every multiple of half a step
    got = run_gpu(A, B, bias, shift, 0)
    want = oracle.gemm_i8(A, B, bias, shift, 0)
    np.testing.assert_array_equal(got, want)
    assert want[0, 129] == 0 and want[0, 131] == 2 and want[0, 127] == 0 and want[0, 125] == -2  # halves go to even


@pytest.mark.parametrize("tile", [None, 256, 192, 128, 64, 32, 320])
def test_sums_around_the_clamp_bounds_and_the_ends_of_int32(tile):
    """The output stage clamps the sums on the way into the rounding shift: sums at and next to the largest one that
    still rounds to 127, the smallest that still rounds to -128, zero, every tie next to them, and the ends of int32,
    on every kernel family (A = 0, so a sum is its bias)."""
    M, N, K = 256, (128 if tile == 320 else 512), 128  # the weight-stationary kernel takes narrow outputs
    A = np.zeros((M, K), np.int8)
    B = np.ones((K, N), np.int8)
    for shift in (1, 2, 9, 10, 16, 17, 18, 23):  # the output stage rounds in fp32 up to 17 and in integers beyond
        half = 1 << (shift - 1)
        centres = [(127 << shift) + half - 1, 127 << shift, (126 << shift) + half, -(128 << shift), -(128 << shift) - half, -(127 << shift) - half,
                   0, half, -half, 3 * half, -3 * half, 2**31 - 1, -(2**31), 2**30, -(2**30)]
        vals = np.array([c + d for c in centres for d in (-2, -1, 0, 1, 2)], dtype=np.int64)
        bias = np.resize(np.clip(vals, -(2**31), 2**31 - 1), N).astype(np.int32)
        for act in (0, 1):
            want = oracle.gemm_i8(A, B, bias, shift, act)
            if tile is None:
                got = run_gpu(A, B, bias, shift, act)
            else:
                C = torch.full((M, N), 77, dtype=torch.int8, device="cuda")
                ops.ac_gemm_i8_planned(dev(A), dev(B), dev(bias), C, shift, act, tile, 1)
                torch.cuda.synchronize()
                got = host(C)
            np.testing.assert_array_equal(got, want)


def test_bias_matrix_and_no_bias():
    A, B, bias = inputs.gemm_i8_inputs(150, 130, 90, seed=5, bias_matrix=True)
    check(A, B, bias, 8, 1)
    check(A, B, None, 8, 1)


@pytest.mark.parametrize("M,N,K", [(64, 64, 8192), (100, 192, 8192), (49, 512, 9216), (17, 16, 8208), (130, 80, 8400)])
def test_split_k_shapes(M, N, K):
    """Few output tiles and a deep K: with a workspace the K range is sliced; results stay bit-exact."""
    assert ops.ac_gemm_i8_workspace_bytes(M, N, K) > 0
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + K)
    check(A, B, bias, 11, 1, workspace=True)
    A, B, biasm = inputs.gemm_i8_inputs(M, N, K, seed=M + K + 1, bias_matrix=True)
    check(A, B, biasm, 9, 0, workspace=True)
    check(A, B, None, 9, 0, workspace=True)


@pytest.mark.parametrize("M,N,K", [(512, 512, 16384), (256, 200, 40000), (300, 260, 70000), (16, 16, 100000), (384, 384, 16384), (1024, 256, 8192)])
def test_few_tiles_deep_k_auto_plan(M, N, K):
    """Tile and K slices chosen together by the library's cost estimate (big tiles with many slices on very deep K)."""
    tile, splits = ops.ac_gemm_i8_auto_plan(M, N, K)
    assert splits > 1
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + K)
    check(A, B, bias, 14, 1, workspace=True)
    check(A, B, None, 16, 0, workspace=True)


def test_k_zero_and_empty():
    bias = np.arange(-40, 40, dtype=np.int32) * 100
    A = np.zeros((5, 0), np.int8)
    B = np.zeros((0, 80), np.int8)
    C = torch.zeros((5, 80), dtype=torch.int8, device="cuda")
    bias_d = dev(bias)
    st = ops.lib().ac_gemm_i8(None, 0, None, 80, bias_d.data_ptr(), 0, C.data_ptr(), 80, 5, 80, 0, 3, 0, None, 0, None)
    assert st == 0
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C), oracle.gemm_i8(A, B, bias, 3, 0))
    # M == 0 or N == 0: accepted, nothing written
    assert ops.lib().ac_gemm_i8(None, 4, None, 0, None, 0, None, 0, 0, 0, 4, 3, 0, None, 0, None) == 0
    assert ops.lib().ac_gemm_i8(None, 4, None, 8, None, 0, None, 8, 0, 8, 4, 3, 0, None, 0, None) == 0


def test_strided_views_and_guard_bands():
    # leading dimensions larger than the rows, unaligned base addresses, and untouched padding in C
    M, N, K = 100, 70, 50
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=6)
    Abig = torch.zeros((M, K + 13), dtype=torch.int8, device="cuda")
    Bbig = torch.zeros((K, N + 7), dtype=torch.int8, device="cuda")
    Cbig = torch.full((M + 2, N + 9), 55, dtype=torch.int8, device="cuda")
    Abig[:, 3:3 + K] = dev(A)
    Bbig[:, 5:5 + N] = dev(B)
    Cv = Cbig[1:1 + M, 4:4 + N]
    ops.ac_gemm_i8(Abig[:, 3:3 + K], Bbig[:, 5:5 + N], dev(bias), Cv, 8, 1)
    torch.cuda.synchronize()
    out = host(Cbig)
    np.testing.assert_array_equal(out[1:1 + M, 4:4 + N], oracle.gemm_i8(A, B, bias, 8, 1))
    mask = np.ones_like(out, dtype=bool)
    mask[1:1 + M, 4:4 + N] = False
    assert (out[mask] == 55).all()


@pytest.mark.parametrize("K", [1024, 8192])
def test_full_size_sampled_large(K):
    """Shapes far larger than the workloads (8192 x 8192 x 1024, and the 8192^3 of the benchmark's scale-up line):
    sampled outputs against the oracle."""
    M = N = 8192
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=77)
    got = run_gpu(A, B, bias, 12, 1)
    rng = np.random.default_rng(0)
    r = np.concatenate([rng.integers(0, M, 20000), np.array([0, M - 1, 0, M - 1])])
    c = np.concatenate([rng.integers(0, N, 20000), np.array([0, 0, N - 1, N - 1])])
    want = oracle.gemm_i8_at(A, B, bias, 12, 1, r, c)
    np.testing.assert_array_equal(got[r, c], want)


def test_argument_errors():
    L = ops.lib()
    a = torch.zeros(64, dtype=torch.int8, device="cuda").data_ptr()
    assert L.ac_gemm_i8(a, 4, a + 16, 4, None, 0, a + 32, 4, 4, 4, 4, 32, 0, None, 0, None) == ops.AC_ERR_SHIFT
    assert L.ac_gemm_i8(a, 4, a + 16, 4, None, 0, a + 32, 4, 4, 4, 4, 3, 2, None, 0, None) == ops.AC_ERR_ACT
    assert L.ac_gemm_i8(a, 3, a + 16, 4, None, 0, a + 32, 4, 4, 4, 4, 3, 0, None, 0, None) == ops.AC_ERR_STRIDE
    assert L.ac_gemm_i8(a, 4, a + 16, 4, None, 0, a, 4, 4, 4, 4, 3, 0, None, 0, None) == ops.AC_ERR_ALIAS
    assert L.ac_gemm_i8(a, 4, None, 4, None, 0, a + 32, 4, 4, 4, 4, 3, 0, None, 0, None) == ops.AC_ERR_NULL
    assert L.ac_gemm_i8(a, 4, a + 16, 4, None, 0, a + 32, 4, -1, 4, 4, 3, 0, None, 0, None) == ops.AC_ERR_SHAPE


@pytest.mark.parametrize("M,N,K", [(64, 64, 64), (300, 200, 130), (320, 208, 144), (1792, 1792, 208), (4096, 3072, 64), (12544, 64, 256)])
def test_raw_accumulator_output(M, N, K):
    """ac_gemm_i8_acc32: the int32 accumulator itself (no scaling, no activation), against the oracle's exact sums."""
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + 3 * N + K)
    _, want = oracle.gemm_i8(A, B, bias, 0, 0, return_acc=True)
    C = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    ops.ac_gemm_i8_acc32(dev(A), dev(B), dev(bias), C)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C).astype(np.int64), want)
    # the paper's own GEMM kernel (Appendix D.1): no bias, no activation, scale 1: the int8 result is sat8 of these sums
    C8 = torch.empty((M, N), dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8(dev(A), dev(B), None, C8, 0, ops.AC_ACT_NONE)
    ops.ac_gemm_i8_acc32(dev(A), dev(B), None, C)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C8), np.clip(host(C), -128, 127).astype(np.int8))


def test_cut_k_launch_replayed_from_a_graph():
    """A launch that cuts K (slices into the workspace, then the combining kernel) captured in a graph and replayed:
    three replays on changing inputs, with eager launches of other cut shapes in between, each against the oracle."""
    M, N, K = 49, 2048, 4608
    assert ops.ac_gemm_i8_auto_plan(M, N, K, True)[1] > 1
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=424242)
    dA, dB, dbias = dev(A), dev(B), dev(bias)
    C = torch.full((M, N), 77, dtype=torch.int8, device="cuda")
    ws = torch.full((ops.ac_gemm_i8_workspace_bytes(M, N, K),), 0xC3, dtype=torch.uint8, device="cuda")
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        ops.ac_gemm_i8(dA, dB, dbias, C, 10, ops.AC_ACT_RELU, workspace=ws)  # first launch outside the capture
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            ops.ac_gemm_i8(dA, dB, dbias, C, 10, ops.AC_ACT_RELU, workspace=ws)
        for rep in range(3):
            A2 = np.roll(A, rep + 1, axis=0)
            dA.copy_(dev(A2))
            C.fill_(55)
            torch.cuda.synchronize()
            g.replay()
            s.synchronize()
            np.testing.assert_array_equal(host(C), oracle.gemm_i8(A2, B, bias, 10, ops.AC_ACT_RELU))
            # eager launches of other cut shapes share nothing with the captured one
            check(*inputs.gemm_i8_inputs(16, 512, 4096, seed=rep), 9, ops.AC_ACT_NONE, workspace=True)
