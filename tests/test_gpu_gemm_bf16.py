"""GPU parity: ac_gemm_bf16 against the fp64 oracle.

Tolerances.  The target is a relative Frobenius error <= 1e-3 against the fp64 result on the
bf16-rounded inputs.  bf16 products are exact in fp32 (8 + 8 significant bits), so the only error is
fp32 accumulation: each of the K additions contributes at most 2^-24 relative to the running sum,
giving |err| <= K * 2^-24 * sum_k |a_k b_k| per element; the element-wise check uses 4x that bound so
a single wrong tile cannot hide inside the norm."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import check_bf16_product_in_full, dev, host, rel_fro
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu
REL_FRO_TOL = 1e-3


def run_gpu(A, B, alpha=1.0, beta=0.0, C_in=None):
    M, K = A.shape
    N = B.shape[1]
    if C_in is None:
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")  # beta == 0 must not read C
    else:
        C = dev(C_in).clone()
    ops.ac_gemm_bf16(dev(A), dev(B), C, alpha, beta)
    torch.cuda.synchronize()
    return host(C)


def check_full(A, B, alpha=1.0, beta=0.0, C_in=None):
    got = run_gpu(A, B, alpha, beta, C_in)
    want = oracle.gemm_bf16(A, B, alpha, beta, C_in)
    assert np.isfinite(got).all()
    assert rel_fro(got, want) <= REL_FRO_TOL
    K = A.shape[1]
    Aa = np.abs(inputs.bf16_bits_to_f32(A).astype(np.float64))
    Ba = np.abs(inputs.bf16_bits_to_f32(B).astype(np.float64))
    bound = 4.0 * (K + 2) * 2.0 ** -24 * (abs(alpha) * (Aa @ Ba) + (abs(beta) * np.abs(C_in) if C_in is not None else 0.0)) + 1e-30
    assert (np.abs(got - want) <= bound).all()
    return got


@pytest.mark.parametrize("M,N,K", [
    (1, 1, 1), (5, 3, 7), (64, 64, 64), (70, 90, 50), (128, 128, 256), (130, 136, 264), (257, 300, 129),
    (1792, 1792, 96), (1800, 1796, 100), (4096, 3072, 64), (4100, 3080, 40), (513, 48, 1000)])
def test_shapes_full_oracle(M, N, K):
    A, B = inputs.gemm_bf16_inputs(M, N, K, seed=M + N + K)
    check_full(A, B)


@pytest.mark.parametrize("M,N,K,plan", [
    (256, 256, 8192, (64, 8)), (128, 128, 262144, (128, 128)), (384, 384, 16384, None), (768, 768, 8192, None),
    (256, 256, 65536, None), (200, 120, 40000, None), (1024, 256, 8192, None)])
def test_few_tiles_deep_k_auto_plan(M, N, K, plan):
    """Few output tiles and a deep K: the library picks tile and K slices from its cost estimate (slices add
    into C with fp32 atomics, so the order of the K / slices partial sums varies from run to run)."""
    auto = ops.ac_gemm_bf16_auto_plan(M, N, K)
    if plan is not None:
        assert auto == plan
    assert auto[1] > 1
    A, B = inputs.gemm_bf16_inputs(M, N, K, seed=M + N + K)
    check_full(A, B)
    C_in = np.random.default_rng(K).standard_normal((M, N)).astype(np.float32)
    check_full(A, B, 0.5, -1.5, C_in)


@pytest.mark.parametrize("M,N,K", [(256, 256, 65536), (200, 120, 40000), (64, 64, 100000), (1024, 256, 8192)])
def test_workspace_call_sums_slices_in_a_fixed_order(M, N, K):
    """ac_gemm_bf16_ws with the workspace it asks for: the oracle's result within the bound, the same bits on
    every run, and the same bits as the planned call on the library's own plan."""
    tile, splits = ops.ac_gemm_bf16_auto_plan(M, N, K)
    need = ops.ac_gemm_bf16_workspace_bytes(M, N, K)
    assert splits > 1 and need == splits * M * N * 4
    A, B = inputs.gemm_bf16_inputs(M, N, K, seed=M + N + K + 1)
    C_in = np.random.default_rng(K).standard_normal((M, N)).astype(np.float32)
    want = oracle.gemm_bf16(A, B, 0.5, -1.5, C_in)
    Ad, Bd = dev(A), dev(B)
    ws = torch.full((need + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    runs = []
    for _ in range(3):
        C = dev(C_in).clone()
        ops.ac_gemm_bf16_ws(Ad, Bd, C, 0.5, -1.5, workspace=ws[:need])
        torch.cuda.synchronize()
        runs.append(host(C))
    assert rel_fro(runs[0], want) <= 1e-3
    np.testing.assert_array_equal(runs[1], runs[0])
    np.testing.assert_array_equal(runs[2], runs[0])
    assert bool((ws[need:] == 0xA5).all())  # nothing written beyond the reported size
    C = dev(C_in).clone()
    ops.ac_gemm_bf16_planned(Ad, Bd, C, 0.5, -1.5, tile, splits, workspace=ws[:need])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C), runs[0])
    # without a workspace the call is ac_gemm_bf16 (atomic adds): same result up to the summation order
    C = dev(C_in).clone()
    ops.ac_gemm_bf16_ws(Ad, Bd, C, 0.5, -1.5)
    torch.cuda.synchronize()
    assert rel_fro(host(C), want) <= 1e-3


def test_workspace_call_on_shapes_that_are_not_cut():
    """A shape with many tiles, and operands the direct-to-LDS kernels do not take: the workspace stays unused and
    the result is ac_gemm_bf16's, bit for bit."""
    for M, N, K, cut in [(512, 512, 256, False), (130, 124, 40004, True)]:
        A, B = inputs.gemm_bf16_inputs(M, N, K, seed=M + K)
        Ad, Bd = dev(A), dev(B)
        need = ops.ac_gemm_bf16_workspace_bytes(M, N, K)
        assert (need > 0) == cut
        ws = torch.full((max(need, 1024),), 0x5A, dtype=torch.uint8, device="cuda")
        C1 = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        C2 = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        ops.ac_gemm_bf16_ws(Ad, Bd, C1, 1.0, 0.0, workspace=ws)
        ops.ac_gemm_bf16(Ad, Bd, C2, 1.0, 0.0)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(C1), host(C2))
        assert bool((ws == 0x5A).all())
        assert rel_fro(host(C1), oracle.gemm_bf16(A, B)) <= 1e-3


def test_alpha_beta():
    A, B = inputs.gemm_bf16_inputs(200, 264, 136, seed=1)
    Cin = np.random.default_rng(2).standard_normal((200, 264)).astype(np.float32)
    check_full(A, B, alpha=0.5, beta=-1.25, C_in=Cin)
    check_full(A, B, alpha=-2.0, beta=0.0)
    got = run_gpu(A, B, alpha=0.0, beta=2.0, C_in=Cin)
    np.testing.assert_array_equal(got, 2.0 * Cin)
    # K == 0: C = beta * C
    C = dev(Cin).clone()
    assert ops.lib().ac_gemm_bf16(None, 0, None, 264, C.data_ptr(), 264, 200, 264, 0, 1.0, 0.5, None) == 0
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C), np.float32(0.5) * Cin)


def test_bit_exact_cases():
    rng = np.random.default_rng(3)
    # small integers: every partial sum is exact in fp32, so any summation order must give the same bits
    Ai = rng.integers(-8, 9, size=(192, 320)).astype(np.float32)
    Bi = rng.integers(-8, 9, size=(320, 160)).astype(np.float32)
    got = run_gpu(inputs.f32_to_bf16_bits(Ai), inputs.f32_to_bf16_bits(Bi))
    np.testing.assert_array_equal(got, (Ai.astype(np.float64) @ Bi.astype(np.float64)).astype(np.float32))
    # K == 1: a product of two bf16 values is exact in fp32
    a, b = inputs.gemm_bf16_inputs(150, 170, 1, seed=4)
    np.testing.assert_array_equal(run_gpu(a, b), oracle.gemm_bf16(a, b).astype(np.float32))
    # identity
    _, Bn = inputs.gemm_bf16_inputs(128, 200, 128, seed=5)
    eye = inputs.f32_to_bf16_bits(np.eye(128, dtype=np.float32))
    np.testing.assert_array_equal(run_gpu(eye, Bn), inputs.bf16_bits_to_f32(Bn))


def test_strided_views_and_guard_bands():
    M, N, K = 90, 70, 40
    A, B = inputs.gemm_bf16_inputs(M, N, K, seed=6)
    Abig = torch.zeros((M, K + 5), dtype=torch.bfloat16, device="cuda")
    Bbig = torch.zeros((K, N + 3), dtype=torch.bfloat16, device="cuda")
    Cbig = torch.full((M + 2, N + 6), 7.0, dtype=torch.float32, device="cuda")
    Abig[:, 1:1 + K] = dev(A)
    Bbig[:, 2:2 + N] = dev(B)
    ops.ac_gemm_bf16(Abig[:, 1:1 + K], Bbig[:, 2:2 + N], Cbig[1:1 + M, 3:3 + N])
    torch.cuda.synchronize()
    out = host(Cbig)
    assert rel_fro(out[1:1 + M, 3:3 + N], oracle.gemm_bf16(A, B)) <= REL_FRO_TOL
    mask = np.ones_like(out, dtype=bool)
    mask[1:1 + M, 3:3 + N] = False
    assert (out[mask] == 7.0).all()


@pytest.mark.parametrize("case", inputs.GEMM_BF16, ids=lambda c: c.name)
def test_workload_configs_in_full(case):
    """Full-size workloads as the benchmark launches them: every output element against the oracle (norm and
    element-wise bound), plus a whole-matrix property, C v == A (B v), evaluated in fp64."""
    A, B = inputs.gemm_bf16_case_inputs(case)
    got = run_gpu(A, B)
    check_bf16_product_in_full(A, B, got)
    rng = np.random.default_rng(0)
    Ad = inputs.bf16_bits_to_f32(A).astype(np.float64)
    Bd = inputs.bf16_bits_to_f32(B).astype(np.float64)
    v = rng.standard_normal((case.N, 3))
    assert rel_fro(got.astype(np.float64) @ v, Ad @ (Bd @ v)) <= 1e-4


def test_argument_errors():
    L = ops.lib()
    a = torch.zeros(1024, dtype=torch.float32, device="cuda").data_ptr()
    assert L.ac_gemm_bf16(a, 4, a + 64, 3, a + 128, 4, 4, 4, 4, 1.0, 0.0, None) == ops.AC_ERR_STRIDE
    assert L.ac_gemm_bf16(a, 4, a + 64, 4, a, 4, 4, 4, 4, 1.0, 0.0, None) == ops.AC_ERR_ALIAS
    assert L.ac_gemm_bf16(a, 4, a + 64, 4, None, 4, 4, 4, 4, 1.0, 0.0, None) == ops.AC_ERR_NULL
    assert L.ac_gemm_bf16(a, 4, a + 64, 4, a + 128, 4, 4, -4, 4, 1.0, 0.0, None) == ops.AC_ERR_SHAPE
    assert L.ac_gemm_bf16(a, 4, a + 64, 4, a + 128, 4, 0, 4, 4, 1.0, 0.0, None) == 0
