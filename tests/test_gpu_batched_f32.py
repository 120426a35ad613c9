"""GPU parity: ac_batched_gemm_f32 against the fp64 oracle (relative Frobenius error <= 1e-5).

fp32 rounding of n <= 16 term sums gives errors near n * 2^-24 ~ 1e-6 relative to the term magnitudes;
the target tolerance of 1e-5 on the Frobenius norm over the whole batch leaves a 10x margin."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host, rel_fro
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu
TOL = 1e-5


def run_gpu(A, B, x=None, d=None, want_C=True):
    batch, n, _ = A.shape
    C = torch.full((batch, n, n), float("nan"), dtype=torch.float32, device="cuda") if want_C else None
    y = torch.full((batch, n), float("nan"), dtype=torch.float32, device="cuda") if x is not None else None
    ops.ac_batched_gemm_f32(dev(A), dev(B), C, dev(x), dev(d), y)
    torch.cuda.synchronize()
    return (host(C) if want_C else None), (host(y) if y is not None else None)


@pytest.mark.parametrize("n,batch", [(12, 1), (12, 31), (12, 32), (12, 37), (12, 4099), (1, 5), (2, 100), (5, 77),
                                     (7, 1001), (8, 64), (15, 33), (16, 130)])
def test_shapes(n, batch):
    A, B, x, d = inputs.batched_f32_inputs(batch, n, seed=n * 1000 + batch)
    Cw, yw = oracle.batched_gemm_f32(A, B, x, d)
    C, y = run_gpu(A, B, x, d)
    assert np.isfinite(C).all() and np.isfinite(y).all()
    assert rel_fro(C, Cw) <= TOL and rel_fro(y, yw) <= TOL
    # element-wise: n products of magnitude <= 1, then n more for y
    assert np.abs(C - Cw).max() <= 4 * n * 2.0 ** -24 * n
    # variants: no add, product only, mat-vec only
    _, y2 = run_gpu(A, B, x, None)
    assert rel_fro(y2, oracle.batched_gemm_f32(A, B, x, None)[1]) <= TOL
    C3, y3 = run_gpu(A, B)
    assert y3 is None and rel_fro(C3, Cw) <= TOL
    C4, y4 = run_gpu(A, B, x, d, want_C=False)
    assert C4 is None and rel_fro(y4, yw) <= TOL


def test_exact_cases():
    n, batch = 12, 50
    A, B, x, d = inputs.batched_f32_inputs(batch, n, seed=9)
    eye = np.broadcast_to(np.eye(n, dtype=np.float32), (batch, n, n)).copy()
    C, y = run_gpu(eye, B, np.zeros_like(x), d)
    np.testing.assert_array_equal(C, B)
    np.testing.assert_array_equal(y, d)
    rng = np.random.default_rng(1)
    Ai = rng.integers(-4, 5, size=(batch, n, n)).astype(np.float32)
    Bi = rng.integers(-4, 5, size=(batch, n, n)).astype(np.float32)
    xi = rng.integers(-4, 5, size=(batch, n)).astype(np.float32)
    di = rng.integers(-4, 5, size=(batch, n)).astype(np.float32)
    C, y = run_gpu(Ai, Bi, xi, di)
    Cw, yw = oracle.batched_gemm_f32(Ai, Bi, xi, di)
    np.testing.assert_array_equal(C, Cw.astype(np.float32))
    np.testing.assert_array_equal(y, yw.astype(np.float32))


def test_workload_config_full():
    case = inputs.BATCHED_F32
    A, B, x, d = inputs.batched_f32_case_inputs(case)
    Cw, yw = oracle.batched_gemm_f32(A, B, x, d)
    C, y = run_gpu(A, B, x, d)
    assert rel_fro(C, Cw) <= TOL and rel_fro(y, yw) <= TOL
    assert np.abs(C - Cw).max() <= 4 * 12 * 2.0 ** -24 * 12


def test_empty_and_errors():
    L = ops.lib()
    a = torch.zeros(4096, dtype=torch.float32, device="cuda").data_ptr()
    assert L.ac_batched_gemm_f32(a, a + 1024, a + 2048, None, None, None, 12, 0, None) == 0
    assert L.ac_batched_gemm_f32(a, a + 1024, a + 2048, None, None, None, 17, 1, None) == ops.AC_ERR_SHAPE
    assert L.ac_batched_gemm_f32(a, a + 1024, a + 2048, None, None, None, 0, 1, None) == ops.AC_ERR_SHAPE
    assert L.ac_batched_gemm_f32(a, a + 1024, None, None, None, None, 12, 1, None) == ops.AC_ERR_NULL
    assert L.ac_batched_gemm_f32(a, a + 1024, a + 2048, a + 3072, None, None, 12, 1, None) == ops.AC_ERR_NULL
    assert L.ac_batched_gemm_f32(a, a + 1024, a, None, None, None, 12, 1, None) == ops.AC_ERR_ALIAS
    assert L.ac_batched_gemm_f32(None, a + 1024, a + 2048, None, None, None, 12, 1, None) == ops.AC_ERR_NULL
