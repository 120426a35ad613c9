"""Helpers shared by the GPU parity tests (device upload, error norms)."""
import numpy as np
import torch


def dev(a):
    """numpy -> device tensor; uint16 arrays are taken as bf16 bit patterns."""
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def rel_fro(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.linalg.norm(want.ravel())
    num = np.linalg.norm((got - want).ravel())
    return num / den if den > 0 else num


def check_bf16_product_in_full(A_bits, B_bits, got, block_rows=2048):
    """Every element of got (fp32, M x N) against the fp64 oracle of the bf16 product A . B, in blocks of rows so
    that the fp64 copies stay small: relative Frobenius error <= 1e-3 over the whole matrix, and element by element
    |err| <= 4 (K + 2) 2^-24 sum_k |a_k b_k| (fp32 accumulation in any order)."""
    import oracle
    from paper_2505_18574_amd import inputs

    M, K = A_bits.shape
    num = den = 0.0
    Ba = np.abs(inputs.bf16_bits_to_f32(B_bits).astype(np.float64))
    for r0 in range(0, M, block_rows):
        r1 = min(M, r0 + block_rows)
        want = oracle.gemm_bf16(A_bits[r0:r1], B_bits)
        g = got[r0:r1].astype(np.float64)
        assert np.isfinite(g).all()
        err = np.abs(g - want)
        mag = np.abs(inputs.bf16_bits_to_f32(A_bits[r0:r1]).astype(np.float64)) @ Ba
        bad = err > 4.0 * (K + 2) * 2.0 ** -24 * mag + 1e-30
        assert not bad.any(), f"rows {r0}..{r1}: {int(bad.sum())} elements beyond the bound, first at {np.argwhere(bad)[0]}"
        num += float((err * err).sum())
        den += float((want * want).sum())
    assert np.sqrt(num) <= 1e-3 * np.sqrt(den)
