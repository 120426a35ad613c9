"""GPU parity on the GEMM shapes the paper names outside its main sweep (Section 5 Table 2, Appendix A
Tables 3 and 5, Appendix D.1), launched as the benchmark's supplementary lines launch them.

int8: the whole output, bit for bit.  bf16: every element against the fp64 oracle with the element-wise bound
4 (K + 2) 2^-24 sum_k |a_k b_k| (fp32 accumulation in any order, K-split slices included), in blocks of rows."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import check_bf16_product_in_full, dev, host, rel_fro
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
def test_bf16_paper_shapes_in_full(case):
    print(case.name, flush=True)
    A, B = inputs.gemm_bf16_case_inputs(case)
    M, N, K = case.M, case.N, case.K
    Ad, Bd = dev(A), dev(B)
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ops.ac_gemm_bf16(Ad, Bd, C)
    torch.cuda.synchronize()
    block = max(64, min(M, (1 << 24) // N))  # fp64 blocks of 128 MB
    check_bf16_product_in_full(A, B, host(C), block)
    # the form the benchmark times: a cut K range summed through a workspace (the uncut shapes run the same kernel)
    need = ops.ac_gemm_bf16_workspace_bytes(M, N, K)
    if need:
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        C.fill_(float("nan"))
        ops.ac_gemm_bf16_ws(Ad, Bd, C, 1.0, 0.0, workspace=ws)
        torch.cuda.synchronize()
        check_bf16_product_in_full(A, B, host(C), block)
