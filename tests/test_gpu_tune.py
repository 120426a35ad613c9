"""GPU parity of the planned launches (every tile / K-split candidate against the oracle) and of the plan
search built on them (Section 3.3: correctness gate first, then latency; Sections 3.5 / 5: schedule reuse)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host, rel_fro
from paper_2505_18574_amd import inputs, ops, tune

pytestmark = pytest.mark.gpu


def workspace_for(M, N, K, plan):
    n = ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, *plan)
    return torch.empty(n, dtype=torch.uint8, device="cuda") if n else None


@pytest.mark.parametrize("M,N,K", [(128, 1024, 1024), (49, 2048, 4608), (300, 272, 656), (512, 768, 768), (64, 64, 16)])
def test_every_int8_plan_is_bit_exact(M, N, K):
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=M + N + K)
    want = oracle.gemm_i8(A, B, bias, 10, 1)
    Ad, Bd, bd = dev(A), dev(B), dev(bias)
    plans = tune.all_plans("i8", M, N, K)
    assert len(plans) >= 3
    for plan in plans:
        print("plan", plan, flush=True)
        C = torch.full((M, N), 55, dtype=torch.int8, device="cuda")
        ops.ac_gemm_i8_planned(Ad, Bd, bd, C, 10, 1, plan[0], plan[1], workspace=workspace_for(M, N, K, plan))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(C), want, err_msg=f"plan {plan}")


def test_int8_plan_with_matrix_bias_and_odd_split():
    M, N, K = 100, 48, 2000
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=77, bias_matrix=True)
    want = oracle.gemm_i8(A, B, bias, 9, 0)
    for plan in [(64, 3), (128, 5), (256, 7), (64, 16)]:
        C = torch.zeros((M, N), dtype=torch.int8, device="cuda")
        ops.ac_gemm_i8_planned(dev(A), dev(B), dev(bias), C, 9, 0, plan[0], plan[1], workspace=workspace_for(M, N, K, plan))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(C), want, err_msg=f"plan {plan}")


@pytest.mark.parametrize("M,N,K", [(256, 256, 8192), (100, 72, 4104), (512, 384, 1024)])
def test_every_bf16_plan_within_bound(M, N, K):
    A, B = inputs.gemm_bf16_inputs(M, N, K, seed=M + K)
    rng = np.random.default_rng(5)
    C_in = rng.standard_normal((M, N)).astype(np.float32)
    Aa = np.abs(inputs.bf16_bits_to_f32(A).astype(np.float64))
    Ba = np.abs(inputs.bf16_bits_to_f32(B).astype(np.float64))
    for alpha, beta in ((1.0, 0.0), (-0.5, 2.0)):
        want = oracle.gemm_bf16(A, B, alpha, beta, C_in if beta else None)
        bound = 4.0 * (K + 2) * 2.0 ** -24 * (abs(alpha) * (Aa @ Ba) + abs(beta) * np.abs(C_in)) + 1e-30
        for plan in tune.all_plans("bf16", M, N, K):
            for with_ws in (False, True):  # slices added into C with atomics / summed through a workspace
                print("plan", plan, alpha, beta, with_ws, flush=True)
                nbytes = ops.ac_gemm_bf16_planned_workspace_bytes(M, N, K, *plan) if with_ws else 0
                ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda") if nbytes else None
                C = dev(C_in).clone() if beta else torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
                ops.ac_gemm_bf16_planned(dev(A), dev(B), C, alpha, beta, plan[0], plan[1], workspace=ws)
                torch.cuda.synchronize()
                got = host(C)
                assert rel_fro(got, want) <= 1e-3, plan
                assert (np.abs(got - want) <= bound).all(), plan
                if with_ws and nbytes:  # the workspace path sums in slice order: two runs agree bit for bit
                    C2 = dev(C_in).clone() if beta else torch.empty((M, N), dtype=torch.float32, device="cuda")
                    ops.ac_gemm_bf16_planned(dev(A), dev(B), C2, alpha, beta, plan[0], plan[1], workspace=ws)
                    torch.cuda.synchronize()
                    assert torch.equal(C, C2), plan


def test_split_refused_for_operands_off_the_fast_path():
    A = torch.zeros((64, 1000), dtype=torch.int8, device="cuda")  # K not a multiple of 16
    B = torch.zeros((1000, 64), dtype=torch.int8, device="cuda")
    C = torch.zeros((64, 64), dtype=torch.int8, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(ops.AcError) as e:
        ops.ac_gemm_i8_planned(A, B, None, C, 0, 0, 64, 2, workspace=ws)
    assert e.value.status == ops.AC_ERR_PLAN
    ops.ac_gemm_i8_planned(A, B, None, C, 0, 0, 64, 1)  # the unsplit plan runs on the generic kernel
    torch.cuda.synchronize()


def test_search_int8_with_oracle_gate_and_reuse():
    """Beam search from the library's own plan, then reuse of the recorded plan on the two reuse targets of
    the row-dominant family (Section 5, Table 2); the gate is the oracle, so every timed candidate is exact."""
    book = tune.PlanBook()
    base, *targets = [inputs.GEMM_I8_PAPER[i] for i in inputs.GEMM_I8_REUSE_FAMILIES[2]]
    for case in (base, *targets):
        A, B, bias = inputs.gemm_i8_case_inputs(case)
        want = torch.from_numpy(oracle.gemm_i8(A, B, bias, case.shift, case.act)).cuda()
        C = torch.empty((case.M, case.N), dtype=torch.int8, device="cuda")
        gate = lambda got: bool(torch.equal(got, want))
        start = book.related("i8", case.M, case.N, case.K) or None
        res = tune.tune_gemm_i8(dev(A), dev(B), dev(bias), C, case.shift, case.act, gate=gate, start=start, iterations=2 if start else 4)
        print(case.name, "best", res.best, f"{res.best_us:.2f} us", [(t.plan, t.correct, t.us and round(t.us, 2)) for t in res.trials], flush=True)
        assert all(t.correct for t in res.trials)
        auto = tune.normalise("i8", case.K, ops.ac_gemm_i8_auto_plan(case.M, case.N, case.K, True))
        if start is None:
            assert auto in [t.plan for t in res.trials]
        assert res.best_us <= min(t.us for t in res.trials) + 1e-9
        book.record("i8", case.M, case.N, case.K, res.best)
        # the winner, run once more, still matches the oracle
        ops.ac_gemm_i8_planned(dev(A), dev(B), dev(bias), C.zero_(), case.shift, case.act, *res.best,
                               workspace=workspace_for(case.M, case.N, case.K, res.best))
        torch.cuda.synchronize()
        assert torch.equal(C, want)
    assert len(book.plans) == 3


@pytest.mark.parametrize("Nb,H,W,Cin,Cout,stride,pad", [(16, 56, 56, 64, 64, 1, 1), (8, 28, 28, 128, 256, 2, 1), (4, 14, 14, 256, 64, 1, 1)])
def test_search_conv_exhaustive_with_oracle_gate(Nb, H, W, Cin, Cout, stride, pad):
    """Every kernel / tile / K split the library offers for a convolution, gated by the oracle: each plan either
    is refused by the library (a geometry its kernel does not take) or reproduces the oracle bit for bit."""
    x, w, bias = inputs.conv_i8_inputs(Nb, H, W, Cin, Cout, 3, 3, seed=Nb + Cin)
    want = torch.from_numpy(oracle.conv2d_i8(x, w, bias, stride, pad, 9, 1)).cuda()
    out = torch.empty_like(want)
    gate = lambda got: bool(torch.equal(got, want))
    res = tune.tune_conv2d_i8(dev(x), dev(w), dev(bias), out, stride, pad, 9, 1, gate=gate, exhaustive=True)
    print("conv", (Nb, H, W, Cin, Cout, stride), "best", res.best, f"{res.best_us:.2f} us",
          [(t.plan, t.us and round(t.us, 2)) for t in res.trials], flush=True)
    M, N, K = want.shape[0] * want.shape[1] * want.shape[2], Cout, 9 * Cin
    assert len(res.trials) == len(tune.all_plans("conv", M, N, K))
    refused = [t.plan for t in res.trials if not t.correct]
    for plan in refused:  # a candidate that is not correct must be one the library refuses, never a wrong result
        with pytest.raises(ops.AcError):
            ops.ac_conv2d_i8(dev(x), dev(w), dev(bias), out, stride, pad, 9, 1, plan=plan)
    assert all(p[0] in tune.WS_TILES + tune.HALO_TILES for p in refused)
    # beam search from the library's own plan ends at a plan no slower than the library's
    res2 = tune.tune_conv2d_i8(dev(x), dev(w), dev(bias), out, stride, pad, 9, 1, gate=gate)
    assert res2.best in [t.plan for t in res.trials]


def test_search_bf16_exhaustive_default_gate():
    M, N, K = 256, 256, 16384
    A, B = inputs.gemm_bf16_inputs(M, N, K, seed=9)
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    res = tune.tune_gemm_bf16(dev(A), dev(B), C, exhaustive=True)
    print("bf16", (M, N, K), "best", res.best, f"{res.best_us:.2f} us", [(t.plan, t.us and round(t.us, 2)) for t in res.trials], flush=True)
    assert all(t.correct for t in res.trials) and len(res.trials) == len(tune.all_plans("bf16", M, N, K))
    nbytes = ops.ac_gemm_bf16_planned_workspace_bytes(M, N, K, *res.best)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda") if nbytes else None
    ops.ac_gemm_bf16_planned(dev(A), dev(B), C, 1.0, 0.0, *res.best, workspace=ws)
    torch.cuda.synchronize()
    assert rel_fro(host(C), oracle.gemm_bf16(A, B)) <= 1e-3
