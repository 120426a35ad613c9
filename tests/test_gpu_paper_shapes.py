"""GPU parity on the GEMM shapes the paper names outside its main sweep (Section 5 Table 2, Appendix A
Tables 3 and 5, Appendix D.1), launched as the benchmark's supplementary lines launch them.

int8: the whole output, bit for bit.  bf16: sampled elements and whole rows against the fp64 oracle with the
element-wise bound 4 (K + 2) 2^-24 sum_k |a_k b_k| (fp32 accumulation in any order, K-split slices included)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host, rel_fro
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", inputs.GEMM_I8_PAPER, ids=lambda c: c.name)
def test_int8_paper_shapes_bit_exact(case):
    A, B, bias = inputs.gemm_i8_case_inputs(case)
    want = oracle.gemm_i8(A, B, bias, case.shift, case.act)
    Ad, Bd, bd = dev(A), dev(B), dev(bias)
    for with_ws in (False, True):
        C = torch.full((case.M, case.N), 77, dtype=torch.int8, device="cuda")
        nbytes = ops.ac_gemm_i8_workspace_bytes(case.M, case.N, case.K) if with_ws else 0
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda") if nbytes else None
        ops.ac_gemm_i8(Ad, Bd, bd, C, case.shift, case.act, workspace=ws)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(C), want)


@pytest.mark.parametrize("case", inputs.GEMM_BF16_PAPER, ids=lambda c: c.name)
def test_bf16_paper_shapes_sampled(case):
    print(case.name, flush=True)
    A, B = inputs.gemm_bf16_case_inputs(case)
    M, N, K = case.M, case.N, case.K
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ops.ac_gemm_bf16(dev(A), dev(B), C)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(C).all())
    rng = np.random.default_rng(1)
    nrand = 6000 if K <= 16384 else 1500
    nrows = 2 if N * K <= (1 << 27) else 0  # whole rows only where the oracle finishes in seconds
    r = np.concatenate([rng.integers(0, M, nrand), [0, 0, M - 1, M - 1], np.repeat(rng.integers(0, M, nrows), N)])
    c = np.concatenate([rng.integers(0, N, nrand), [0, N - 1, 0, N - 1], np.tile(np.arange(N), nrows)])
    want, mag = oracle.gemm_bf16_at(A, B, r, c)
    g = host(C[torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()]).astype(np.float64)
    assert rel_fro(g, want) <= 1e-3
    assert (np.abs(g - want) <= 4.0 * (K + 2) * 2.0 ** -24 * mag + 1e-30).all()
    # whole-matrix property on the device output: column sums of C against A^T-weighted sums in fp64
    ones = torch.ones(M, dtype=torch.float64, device="cuda")
    colsum = host(ones @ C.double())
    Ad = inputs.bf16_bits_to_f32(A).astype(np.float64)
    Bd = inputs.bf16_bits_to_f32(B).astype(np.float64)
    assert rel_fro(colsum, Ad.sum(axis=0) @ Bd) <= 1e-4
    # the form the benchmark times: a cut K range summed through a workspace (the uncut shapes run the same kernel)
    need = ops.ac_gemm_bf16_workspace_bytes(M, N, K)
    if need:
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        C2 = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        ops.ac_gemm_bf16_ws(dev(A), dev(B), C2, 1.0, 0.0, workspace=ws)
        torch.cuda.synchronize()
        g2 = host(C2[torch.from_numpy(r).cuda(), torch.from_numpy(c).cuda()]).astype(np.float64)
        assert rel_fro(g2, want) <= 1e-3
        assert (np.abs(g2 - want) <= 4.0 * (K + 2) * 2.0 ** -24 * mag + 1e-30).all()
        assert rel_fro(host(ones @ C2.double()), Ad.sum(axis=0) @ Bd) <= 1e-4
