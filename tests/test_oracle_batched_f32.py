"""Pins for the batched small fp32 oracle and the TinyMPC forward recurrence (Section 4.4.3, Appendix D.2)."""
import numpy as np
import pytest

import oracle
from conftest import read_golden_table
from paper_2505_18574_amd import inputs


@pytest.mark.parametrize("n,batch", [(12, 37), (1, 5), (4, 16), (16, 3), (7, 9)])
def test_vs_einsum_float64(n, batch):
    A, B, x, d = inputs.batched_f32_inputs(batch, n, seed=41)
    C, y = oracle.batched_gemm_f32(A, B, x, d)
    Cw = np.einsum("bik,bkj->bij", A.astype(np.float64), B.astype(np.float64))
    yw = np.einsum("bij,bj->bi", Cw, x.astype(np.float64)) + d.astype(np.float64)
    np.testing.assert_allclose(C, Cw, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(y, yw, rtol=1e-13, atol=1e-14)
    C2, y2 = oracle.batched_gemm_f32(A, B, x, None)
    np.testing.assert_allclose(y2, yw - d, rtol=1e-12, atol=1e-13)
    C3, y3 = oracle.batched_gemm_f32(A, B)
    assert y3 is None
    np.testing.assert_array_equal(C3, C)


def test_special_cases():
    n, batch = 12, 6
    A, B, x, d = inputs.batched_f32_inputs(batch, n, seed=42)
    eye = np.broadcast_to(np.eye(n, dtype=np.float32), (batch, n, n)).copy()
    C, y = oracle.batched_gemm_f32(eye, B, x, d)
    np.testing.assert_array_equal(C, B.astype(np.float64))
    np.testing.assert_allclose(y, np.einsum("bij,bj->bi", B.astype(np.float64), x.astype(np.float64)) + d, rtol=1e-14)
    C, y = oracle.batched_gemm_f32(A, B, np.zeros_like(x), d)
    np.testing.assert_array_equal(y, d.astype(np.float64))
    # items are independent: permuting the batch permutes the outputs
    p = np.random.default_rng(0).permutation(batch)
    C1, y1 = oracle.batched_gemm_f32(A, B, x, d)
    C2, y2 = oracle.batched_gemm_f32(A[p], B[p], x[p], d[p])
    np.testing.assert_array_equal(C2, C1[p])
    np.testing.assert_array_equal(y2, y1[p])
    # (A B)^T = B^T A^T
    Ct, _ = oracle.batched_gemm_f32(np.ascontiguousarray(B.transpose(0, 2, 1)), np.ascontiguousarray(A.transpose(0, 2, 1)))
    np.testing.assert_allclose(Ct, C1.transpose(0, 2, 1), rtol=1e-13, atol=1e-14)


def test_workload_counts():
    c = inputs.BATCHED_F32
    assert c.ops == 262144 * 3756 and c.bytes == 262144 * 1872


def test_tinympc_scalar_hand_values():
    for row in read_golden_table("tinympc_scalar.txt"):
        h = (len(row) - 4) // 3
        A, B, K, x0 = row[:4]
        d, u, xs = row[4:4 + h], row[4 + h:4 + 2 * h], row[4 + 2 * h:]
        f = lambda v: np.array(v, dtype=np.float32)
        got_u, got_x = oracle.tinympc_forward(f([[A]]), f([[B]]), f([[K]]), f([[x0]]), f(d).reshape(1, h, 1), return_x=True)
        assert got_u.ravel().tolist() == [float(v) for v in u]
        assert got_x.ravel().tolist() == [float(x0)] + [float(v) for v in xs]


def test_tinympc_closed_forms():
    Adyn, Bdyn, Kinf, x0, d = inputs.tinympc_inputs(batch=9, seed=43)
    A64, B64, K64 = Adyn.astype(np.float64), Bdyn.astype(np.float64), Kinf.astype(np.float64)
    u, xs = oracle.tinympc_forward(Adyn, Bdyn, Kinf, x0, d, return_x=True)
    assert u.shape == (9, 5, 4) and xs.shape == (9, 6, 12)
    # closed loop: x[i+1] = (A - B K) x[i] - B d[i], u[i] = -K x[i] - d[i]
    Acl = A64 - B64 @ K64
    x = x0.astype(np.float64)
    for i in range(5):
        np.testing.assert_allclose(xs[:, i], x, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(u[:, i], -(x @ K64.T) - d[:, i], rtol=1e-12, atol=1e-12)
        x = x @ Acl.T - d[:, i].astype(np.float64) @ B64.T
    np.testing.assert_allclose(xs[:, 5], x, rtol=1e-12, atol=1e-12)
    # Bdyn = 0: x[i] = Adyn^i x0
    u0, xs0 = oracle.tinympc_forward(Adyn, np.zeros_like(Bdyn), Kinf, x0, d, return_x=True)
    for i in range(6):
        np.testing.assert_allclose(xs0[:, i], x0.astype(np.float64) @ np.linalg.matrix_power(A64, i).T, rtol=1e-11, atol=1e-12)
    # Kinf = 0: u[i] = -d[i]
    uz = oracle.tinympc_forward(Adyn, Bdyn, np.zeros_like(Kinf), x0, d)
    np.testing.assert_array_equal(uz, -d.astype(np.float64))
