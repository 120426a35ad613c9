"""GPU parity: ac_tinympc_forward_f32 against the fp64 oracle of the printed recurrence (Appendix D.2).

fp32 sums of at most nx + nu terms per element and `horizon` dependent steps (fused multiply-add chains, or for the
paper's sizes 16 x 16 products on the matrix units with u substituted into the state update): rounding stays near
1e-6 relative to the magnitudes involved, so the bar is the fp32 one of the library (relative Frobenius error
<= 1e-5 over the batch).  Both kernel families are covered: (12, 4) with aligned arrays takes the matrix units (horizon
5 with whole-run loads and stores, other horizons per lane), everything else the vector ALU."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host, rel_fro
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu
TOL = 1e-5


def run_gpu(Adyn, Bdyn, Kinf, x0, d, want_x):
    batch, horizon, nu = d.shape
    nx = Adyn.shape[0]
    u = torch.full((batch, horizon, nu), float("nan"), dtype=torch.float32, device="cuda")
    xs = torch.full((batch, horizon + 1, nx), float("nan"), dtype=torch.float32, device="cuda") if want_x else None
    ops.ac_tinympc_forward_f32(dev(Adyn), dev(Bdyn), dev(Kinf), dev(x0), dev(d), u, xs)
    torch.cuda.synchronize()
    return host(u), (host(xs) if want_x else None)


@pytest.mark.parametrize("nx,nu,horizon,batch", [(12, 4, 5, 1), (12, 4, 5, 255), (12, 4, 5, 1000), (12, 4, 1, 300), (12, 4, 9, 513),
                                                 (1, 1, 3, 10), (16, 16, 4, 100), (5, 3, 6, 257), (8, 2, 2, 64)])
def test_shapes(nx, nu, horizon, batch):
    Adyn, Bdyn, Kinf, x0, d = inputs.tinympc_inputs(batch, seed=nx * 100 + horizon, nx=nx, nu=nu, horizon=horizon)
    # keep the closed loop from blowing up over long horizons
    Adyn = (Adyn / max(1.0, 0.6 * nx ** 0.5)).astype(np.float32)
    uw, xw = oracle.tinympc_forward(Adyn, Bdyn, Kinf, x0, d, return_x=True)
    u, xs = run_gpu(Adyn, Bdyn, Kinf, x0, d, want_x=True)
    assert np.isfinite(u).all() and np.isfinite(xs).all()
    assert rel_fro(u, uw) <= TOL and rel_fro(xs, xw) <= TOL
    u2, none = run_gpu(Adyn, Bdyn, Kinf, x0, d, want_x=False)
    assert none is None
    np.testing.assert_array_equal(u2, u)


def test_paper_sizes_on_unaligned_arrays():
    """(12, 4, 5) with x0 and u four bytes off a 16-byte boundary: the vector-ALU kernel, same bar."""
    batch, horizon = 333, 5
    Adyn, Bdyn, Kinf, x0, d = inputs.tinympc_inputs(batch, seed=4242)
    Adyn = (Adyn / 2).astype(np.float32)
    uw, xw = oracle.tinympc_forward(Adyn, Bdyn, Kinf, x0, d, return_x=True)
    x0_buf = torch.zeros(batch * 12 + 1, dtype=torch.float32, device="cuda")
    u_buf = torch.full((batch * horizon * 4 + 1,), float("nan"), dtype=torch.float32, device="cuda")
    x0_v, u_v = x0_buf[1:].view(batch, 12), u_buf[1:].view(batch, horizon, 4)
    x0_v.copy_(dev(x0))
    xs = torch.full((batch, horizon + 1, 12), float("nan"), dtype=torch.float32, device="cuda")
    ops.ac_tinympc_forward_f32(dev(Adyn), dev(Bdyn), dev(Kinf), x0_v, dev(d), u_v, xs)
    torch.cuda.synchronize()
    assert rel_fro(host(u_v), uw) <= TOL and rel_fro(host(xs), xw) <= TOL


@pytest.mark.parametrize("horizon,batch", [(3, 77), (5, 77), (5, 700), (5, 64), (5, 65), (5, 1025)])
def test_exact_small_integers(horizon, batch):
    rng = np.random.default_rng(0)
    f = lambda shape, lo, hi: rng.integers(lo, hi + 1, size=shape).astype(np.float32)
    Adyn, Bdyn, Kinf = f((12, 12), -1, 1), f((12, 4), -1, 1), f((4, 12), -1, 1)
    x0, d = f((batch, 12), -2, 2), f((batch, horizon, 4), -2, 2)
    uw, xw = oracle.tinympc_forward(Adyn, Bdyn, Kinf, x0, d, return_x=True)
    assert np.abs(xw).max() < 2 ** 24  # every intermediate is an exactly representable integer
    u, xs = run_gpu(Adyn, Bdyn, Kinf, x0, d, want_x=True)
    np.testing.assert_array_equal(u, uw.astype(np.float32))
    np.testing.assert_array_equal(xs, xw.astype(np.float32))


def test_full_batch():
    Adyn, Bdyn, Kinf, x0, d = inputs.tinympc_inputs(262144, seed=6000)
    Adyn = (Adyn / 2).astype(np.float32)
    uw, xw = oracle.tinympc_forward(Adyn, Bdyn, Kinf, x0, d, return_x=True)
    u, xs = run_gpu(Adyn, Bdyn, Kinf, x0, d, want_x=True)
    assert rel_fro(u, uw) <= TOL and rel_fro(xs, xw) <= TOL
    u2, _ = run_gpu(Adyn, Bdyn, Kinf, x0, d, want_x=False)
    np.testing.assert_array_equal(u2, u)


def test_empty_and_errors():
    L = ops.lib()
    a = torch.zeros(4096, dtype=torch.float32, device="cuda").data_ptr()
    args = (a, a + 1024, a + 2048, a + 3072, a + 4096, a + 5120)
    assert L.ac_tinympc_forward_f32(*args, None, 12, 4, 5, 0, None) == 0
    assert L.ac_tinympc_forward_f32(*args, None, 12, 4, 0, 7, None) == 0
    assert L.ac_tinympc_forward_f32(*args, None, 17, 4, 5, 7, None) == ops.AC_ERR_SHAPE
    assert L.ac_tinympc_forward_f32(*args, None, 12, 0, 5, 7, None) == ops.AC_ERR_SHAPE
    assert L.ac_tinympc_forward_f32(a, a + 1024, a + 2048, a + 3072, a + 4096, None, None, 12, 4, 5, 7, None) == ops.AC_ERR_NULL
    assert L.ac_tinympc_forward_f32(a, a + 1024, a + 2048, a + 3072, a + 4096, a + 4096, None, 12, 4, 5, 7, None) == ops.AC_ERR_ALIAS
