"""GPU parity where byte offsets leave 32 bits: outputs larger than 4 GiB (sampled rows on both sides of the
2^31 and 2^32 byte marks, checked against the oracle) and operand row pitches so long that 256 rows span more
than 4 GiB (such operands take the kernels whose lanes carry 64-bit addresses)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host, rel_fro
from paper_2505_18574_amd import inputs, ops

pytestmark = pytest.mark.gpu


def sample_rows(M, row_bytes, seed):
    """First and last rows, the rows next to the 2^31 and 2^32 byte offsets, and a random handful."""
    rows = {0, 1, M - 2, M - 1}
    for mark in (1 << 31, 1 << 32):
        r = mark // row_bytes
        rows.update(x for x in (r - 1, r, r + 1) if 0 <= x < M)
    rows.update(int(x) for x in np.random.default_rng(seed).integers(0, M, 24))
    return np.array(sorted(rows), dtype=np.int64)


def test_int8_output_beyond_4_gib():
    M, N, K, shift = 70000, 65536, 32, 5
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=9100)
    C = torch.full((M, N), 91, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8(dev(A), dev(B), dev(bias), C, shift, 1)
    torch.cuda.synchronize()
    rows = sample_rows(M, N, 1)
    assert rows.max() * N >= 1 << 32
    want = oracle.gemm_i8(A[rows], B, bias, shift, 1)
    np.testing.assert_array_equal(host(C[torch.from_numpy(rows).cuda()]), want)


def test_int32_accumulator_output_beyond_4_gib():
    M, N, K = 40000, 32768, 32
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=9101)
    C = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    ops.ac_gemm_i8_acc32(dev(A), dev(B), dev(bias), C)
    torch.cuda.synchronize()
    rows = sample_rows(M, 4 * N, 2)
    assert rows.max() * 4 * N >= 1 << 32
    _, want = oracle.gemm_i8(A[rows], B, bias, 0, 0, return_acc=True)
    np.testing.assert_array_equal(host(C[torch.from_numpy(rows).cuda()]).astype(np.int64), want)


def test_bf16_output_beyond_4_gib():
    M, N, K = 40000, 32768, 32
    A, B = inputs.gemm_bf16_inputs(M, N, K, seed=9102)
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ops.ac_gemm_bf16(dev(A), dev(B), C, 1.0, 0.0)
    torch.cuda.synchronize()
    rows = sample_rows(M, 4 * N, 3)
    want = oracle.gemm_bf16(A[rows], B)
    got = host(C[torch.from_numpy(rows).cuda()])
    assert rel_fro(got, want) <= 1e-3
    assert np.abs(got - want).max() <= 1e-4 * np.abs(want).max()


def strided(t2d, pitch):
    """The same matrix in rows `pitch` elements apart (the gaps are never read)."""
    rows, cols = t2d.shape
    big = torch.empty(rows * pitch, dtype=t2d.dtype, device="cuda")
    view = big.as_strided((rows, cols), (pitch, 1))
    view.copy_(t2d)
    return view


@pytest.mark.parametrize("which", ["lda", "ldb"])
def test_int8_row_pitch_beyond_32_bit_lane_offsets(which):
    M, N, K, shift = 300, 48, 256, 6
    A, B, bias = inputs.gemm_i8_inputs(M, N, K, seed=9103)
    want = oracle.gemm_i8(A, B, bias, shift, 0)
    Ad = strided(dev(A), (1 << 24) + 16) if which == "lda" else dev(A)   # 256 rows of A span 4 GiB
    Bd = strided(dev(B), (1 << 26) + 16) if which == "ldb" else dev(B)   # 64 rows of B span 4 GiB (256 rows: 17 GB)
    C = torch.full((M, N), 91, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8(Ad, Bd, dev(bias), C, shift, 0)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C), want)
    C32 = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    ops.ac_gemm_i8_acc32(Ad, Bd, dev(bias), C32)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C32).astype(np.int64), oracle.gemm_i8(A, B, bias, 0, 0, return_acc=True)[1])
    # a K split needs the direct-to-LDS kernels, which these operands do not qualify for
    ws = torch.empty(ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, 64, 2), dtype=torch.uint8, device="cuda")
    with pytest.raises(ops.AcError) as err:
        ops.ac_gemm_i8_planned(Ad, Bd, dev(bias), C, shift, 0, 64, 2, workspace=ws)
    assert err.value.status == ops.AC_ERR_PLAN


def test_bf16_row_pitch_beyond_32_bit_lane_offsets():
    M, N, K = 300, 48, 64
    A, B = inputs.gemm_bf16_inputs(M, N, K, seed=9104)
    want = oracle.gemm_bf16(A, B)
    Ad = strided(dev(A), (1 << 23) + 8)   # 16 MiB rows: 256 of them span 4 GiB
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ops.ac_gemm_bf16(Ad, dev(B), C, 1.0, 0.0)
    torch.cuda.synchronize()
    assert rel_fro(host(C), want) <= 1e-3


def sample_items(batch, item_bytes, seed):
    items = {0, 1, 2, 3, batch - 5, batch - 4, batch - 3, batch - 2, batch - 1}
    for mark in (1 << 31, 1 << 32):
        b = mark // item_bytes
        items.update(x for x in range(b - 2, b + 3) if 0 <= x < batch)
    items.update(int(x) for x in np.random.default_rng(seed).integers(0, batch, 200))
    return np.array(sorted(items), dtype=np.int64)


def test_batched_f32_arrays_beyond_4_gib():
    """8 million items of 12 x 12 (A, B and C are 4.6 GB each; a ragged last group), inputs drawn on the device
    from a seeded generator; sampled items against the oracle."""
    batch, n = 8_000_003, 12
    g = torch.Generator(device="cuda").manual_seed(9105)
    u01 = lambda *shape: torch.rand(shape, device="cuda", generator=g) * 2.0 - 1.0
    A, B, x, d = u01(batch, n, n), u01(batch, n, n), u01(batch, n), u01(batch, n)
    C = torch.full((batch, n, n), float("nan"), dtype=torch.float32, device="cuda")
    y = torch.full((batch, n), float("nan"), dtype=torch.float32, device="cuda")
    ops.ac_batched_gemm_f32(A, B, C, x, d, y)
    torch.cuda.synchronize()
    idx = sample_items(batch, 4 * n * n, 4)
    assert idx.max() * 4 * n * n >= 1 << 32
    t = torch.from_numpy(idx).cuda()
    Cw, yw = oracle.batched_gemm_f32(host(A[t]), host(B[t]), host(x[t]), host(d[t]))
    assert rel_fro(host(C[t]), Cw) <= 1e-5 and rel_fro(host(y[t]), yw) <= 1e-5
    assert bool(torch.isfinite(y).all())  # every item was written


def test_tinympc_forward_arrays_beyond_4_gib():
    """15 million problems: the state trajectories are 4.3 GB; sampled problems against the oracle."""
    batch, nx, nu, hz = 15_000_001, 12, 4, 5
    g = torch.Generator(device="cuda").manual_seed(9106)
    u01 = lambda *shape: torch.rand(shape, device="cuda", generator=g) * 2.0 - 1.0
    Ad, Bd, Ki = u01(nx, nx) * 0.3, u01(nx, nu), u01(nu, nx) * 0.3
    x0, dd = u01(batch, nx), u01(batch, hz, nu)
    u = torch.full((batch, hz, nu), float("nan"), dtype=torch.float32, device="cuda")
    xs = torch.full((batch, hz + 1, nx), float("nan"), dtype=torch.float32, device="cuda")
    ops.ac_tinympc_forward_f32(Ad, Bd, Ki, x0, dd, u, xs)
    torch.cuda.synchronize()
    idx = sample_items(batch, 4 * (hz + 1) * nx, 5)
    assert idx.max() * 4 * (hz + 1) * nx >= 1 << 32
    t = torch.from_numpy(idx).cuda()
    uw, xw = oracle.tinympc_forward(host(Ad), host(Bd), host(Ki), host(x0[t]), host(dd[t]), return_x=True)
    assert rel_fro(host(u[t]), uw) <= 1e-5 and rel_fro(host(xs[t]), xw) <= 1e-5
    assert bool(torch.isfinite(u).all())


MAX_DIM = 1 << 29  # the largest dimension the library accepts


def _rows_of(M, row_bytes, seed):
    return torch.from_numpy(sample_rows(M, row_bytes, seed)).cuda()


@pytest.mark.parametrize("N,K", [(16, 16), (12, 10)])
def test_int8_gemm_with_the_largest_row_count(N, K):
    """M = 2^29 (8 million blocks of 64 rows; operands drawn on the device, 8.6 GB each): the library's own plan, two
    named tiles, the int32 accumulator read and the transposed-A form, on sampled rows.  N = 12, K = 10 takes the
    kernels without alignment requirements."""
    M = MAX_DIM
    g = torch.Generator(device="cuda").manual_seed(9107)
    A = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda", generator=g)
    B = torch.randint(-128, 128, (K, N), dtype=torch.int8, device="cuda", generator=g)
    bias = torch.randint(-(1 << 15), 1 << 15, (N,), dtype=torch.int32, device="cuda", generator=g)
    rows = _rows_of(M, N, 6)
    want, acc = oracle.gemm_i8(host(A[rows]), host(B), host(bias), 4, 1, return_acc=True)
    C = torch.full((M, N), 91, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8(A, B, bias, C, 4, 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C[rows]), want)
    if N % 16 == 0 and K % 16 == 0:
        for tile in (64, 256):
            C.fill_(91)
            ops.ac_gemm_i8_planned(A, B, bias, C, 4, 1, tile, 1)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(host(C[rows]), want, err_msg=f"tile {tile}")
    del C
    C32 = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    ops.ac_gemm_i8_acc32(A, B, bias, C32)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C32[rows]).astype(np.int64), acc)
    del C32
    At = A.t().contiguous()  # K x M
    del A
    C = torch.full((M, N), 91, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8_t(At, B, bias, C, 4, 1, trans_a=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C[rows]), want)


def test_int8_one_wave_per_tile_kernel_with_millions_of_tiles():
    """M = 2^27 rows of 64 bytes through tile code 32 by name: 4.2 million tiles (one wave each, a million
    workgroups), row offsets beyond 2^32 bytes in A; sampled rows."""
    M, N, K = 1 << 27, 16, 64
    g = torch.Generator(device="cuda").manual_seed(9108)
    A = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda", generator=g)
    B = torch.randint(-128, 128, (K, N), dtype=torch.int8, device="cuda", generator=g)
    bias = torch.randint(-(1 << 15), 1 << 15, (N,), dtype=torch.int32, device="cuda", generator=g)
    rows = _rows_of(M, N, 7)
    want = oracle.gemm_i8(host(A[rows]), host(B), host(bias), 6, 1)
    C = torch.full((M, N), 91, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8_planned(A, B, bias, C, 6, 1, 32, 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C[rows]), want)


def test_bf16_gemm_with_the_largest_row_count():
    M, N, K = MAX_DIM, 8, 8
    g = torch.Generator(device="cuda").manual_seed(9108)
    A = torch.randn((M, K), device="cuda", generator=g).to(torch.bfloat16)
    B = torch.randn((K, N), device="cuda", generator=g).to(torch.bfloat16)
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ops.ac_gemm_bf16(A, B, C, 1.0, 0.0)
    torch.cuda.synchronize()
    rows = _rows_of(M, 4 * N, 7)
    bits = lambda t: host(t.view(torch.int16)).view(np.uint16)
    want = oracle.gemm_bf16(bits(A[rows]), bits(B))
    assert rel_fro(host(C[rows]), want) <= 1e-3
    assert bool(torch.isfinite(C).all())


def _deep_k_operands(M, N, K, dtype):
    """A[i][k] = +1 / -1 by row, B[k][j] = (k + j) mod 3 - 1: every exact sum has a closed form (no oracle pass over
    2^29 terms), every partial sum stays far inside int32 and is exact in fp32."""
    sign = np.where(np.arange(M) % 2 == 0, 1, -1).astype(np.int64)
    A = torch.from_numpy(sign).to(dtype).cuda()[:, None].expand(M, K).contiguous()
    B = torch.empty((K, N), dtype=dtype, device="cuda")
    step = 1 << 24
    cols = torch.arange(N, device="cuda", dtype=torch.int32)[None, :]
    for k0 in range(0, K, step):
        k = torch.arange(k0, min(K, k0 + step), device="cuda", dtype=torch.int32)[:, None]
        B[k0:k0 + step] = ((k + cols) % 3 - 1).to(dtype)
    # sum_k B[k][j]: residues r = (k + j) mod 3 contribute r - 1, so the sum is (#r == 2) - (#r == 0)
    ks = np.arange(3)
    count = np.array([(K - 1 - ks[r]) // 3 + 1 if ks[r] < K else 0 for r in range(3)], dtype=np.int64)  # k == r mod 3
    colsum = np.array([count[(2 - j) % 3] - count[(0 - j) % 3] for j in range(N)], dtype=np.int64)
    return A, B, sign[:, None] * colsum[None, :]


def test_int8_gemm_with_the_deepest_k():
    """K = 2^29 (four million K tiles) on a 16 x 16 output: cut into slices with a workspace, one workgroup without;
    the expected accumulators come from the closed form and pass through the oracle's output stage."""
    M, N, K = 16, 16, MAX_DIM
    A, B, acc = _deep_k_operands(M, N, K, torch.int8)
    assert np.abs(acc).max() <= 1 and K % 3 != 0  # the three residues nearly cancel: small sums, so add a bias that matters
    bias = (np.arange(N, dtype=np.int64) - 8) * 100000
    want = oracle.requantise_vec(acc + bias[None, :], 12, 0)
    need = ops.ac_gemm_i8_workspace_bytes(M, N, K)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    for workspace in (ws, None):
        C = torch.full((M, N), 91, dtype=torch.int8, device="cuda")
        ops.ac_gemm_i8(A, B, dev(bias.astype(np.int32)), C, 12, 0, workspace=workspace)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(C), want)
    C32 = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    ops.ac_gemm_i8_acc32(A, B, dev(bias.astype(np.int32)), C32)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C32).astype(np.int64), acc + bias[None, :])


def test_bf16_gemm_with_the_deepest_k():
    M, N, K = 16, 16, MAX_DIM
    A, B, acc = _deep_k_operands(M, N, K, torch.bfloat16)
    need = ops.ac_gemm_bf16_workspace_bytes(M, N, K)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    for workspace in (ws, None):
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        ops.ac_gemm_bf16_ws(A, B, C, 1.0, 0.0, workspace=workspace)
        torch.cuda.synchronize()
        # every product is -1, 0 or +1 and the sums of a slice stay below 2^24 in magnitude: fp32 is exact here
        np.testing.assert_array_equal(host(C), acc.astype(np.float32))


def _cols_of(N, seed):
    cols = {0, 1, N - 2, N - 1}
    cols.update(int(x) for x in np.random.default_rng(seed).integers(0, N, 300))
    return np.array(sorted(cols), dtype=np.int64)


@pytest.mark.parametrize("N", [(1 << 25) - 1024, MAX_DIM])
def test_gemms_with_the_widest_outputs(N):
    """A 16-row product with N = 2^25 - 1024 columns (the longest B rows the direct-to-LDS kernels address) and with
    N = 2^29 (the largest the library accepts; rows of B half a gigabyte apart): sampled columns against the oracle
    for the int8 call, the accumulator read and the bf16 call."""
    M, K = 16, 16
    g = torch.Generator(device="cuda").manual_seed(9109)
    A = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda", generator=g)
    B = torch.randint(-128, 128, (K, N), dtype=torch.int8, device="cuda", generator=g)
    bias = torch.randint(-(1 << 15), 1 << 15, (N,), dtype=torch.int32, device="cuda", generator=g)
    cols = _cols_of(N, 8)
    ct = torch.from_numpy(cols).cuda()
    want, acc = oracle.gemm_i8(host(A), host(B[:, ct]), host(bias[ct]), 5, 0, return_acc=True)
    C = torch.full((M, N), 91, dtype=torch.int8, device="cuda")
    ops.ac_gemm_i8(A, B, bias, C, 5, 0)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C[:, ct]), want)
    assert int((C[:, -4096:] == 91).sum()) < 4096  # the last columns were written (a stray 91 is a legitimate value)
    del C
    C32 = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    ops.ac_gemm_i8_acc32(A, B, bias, C32)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(C32[:, ct]).astype(np.int64), acc)
    del C32, B, bias
    Ab = torch.randn((M, K), device="cuda", generator=g).to(torch.bfloat16)
    Bb = torch.empty((K, N), dtype=torch.bfloat16, device="cuda")
    for k in range(K):  # row by row: a whole fp32 draw of B would be 34 GB
        Bb[k] = torch.randn((N,), device="cuda", generator=g).to(torch.bfloat16)
    Cf = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ops.ac_gemm_bf16(Ab, Bb, Cf, 1.0, 0.0)
    torch.cuda.synchronize()
    bits = lambda t: host(t.contiguous().view(torch.int16)).view(np.uint16)
    assert rel_fro(host(Cf[:, ct]), oracle.gemm_bf16(bits(Ab), bits(Bb[:, ct]))) <= 1e-3
    assert bool(torch.isfinite(Cf[:, -4096:]).all())


def test_convolution_on_the_largest_input():
    """An NHWC input of 2^31 - 1 MB elements (2047 images of 128 x 128 x 64; the library takes inputs below 2^31
    elements): the library's own choice and every kernel family by name, on images sampled from both ends and from
    the 2^30 byte mark, against the oracle run on those images alone (images are independent)."""
    Nb, H, W, Cin, Cout = 2047, 128, 128, 64, 16
    g = torch.Generator(device="cuda").manual_seed(9110)
    x = torch.randint(-128, 128, (Nb, H, W, Cin), dtype=torch.int8, device="cuda", generator=g)
    w = torch.randint(-128, 128, (3, 3, Cin, Cout), dtype=torch.int8, device="cuda", generator=g)
    b = torch.randint(-(1 << 15), 1 << 15, (Cout,), dtype=torch.int32, device="cuda", generator=g)
    imgs = torch.tensor([0, 1023, 1024, 2046], device="cuda")
    want = oracle.conv2d_i8(host(x[imgs]), host(w), host(b), 1, 1, 11, 1)
    out = torch.full((Nb, H, W, Cout), 17, dtype=torch.int8, device="cuda")
    M, K = Nb * H * W, 9 * Cin
    ran = 0
    for plan in (None, (64, 1), (256, 1), (192, 1), (320, 1), (321, 1), (64, 2)):
        out.fill_(17)
        need = ops.ac_gemm_i8_planned_workspace_bytes(M, Cout, K, *plan) if plan else ops.ac_gemm_i8_workspace_bytes(M, Cout, K)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
        try:
            ops.ac_conv2d_i8(x, w, b, out, 1, 1, 11, 1, workspace=ws, plan=plan)
        except ops.AcError as e:
            assert plan is not None and e.status == ops.AC_ERR_PLAN, plan
            continue
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(out[imgs]), want, err_msg=f"plan {plan}")
        ran += 1
    assert ran == 7  # this geometry qualifies for every family
    # one more image would pass 2^31 elements: refused before anything is launched
    st = ops.lib().ac_conv2d_i8(x.data_ptr(), w.data_ptr(), b.data_ptr(), out.data_ptr(), Nb + 1, H, W, Cin, Cout, 3, 3, 1, 1, 11, 1, None, 0, None)
    assert st == ops.AC_ERR_SHAPE
