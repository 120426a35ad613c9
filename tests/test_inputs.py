"""The seeded generators: determinism, ranges, and the bf16 rounding of input data."""
import numpy as np
import torch

from paper_2505_18574_amd import inputs


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32),
                        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, -1.0 - 2.0 ** -8, 0.0, -0.0,
                                  3.0e38, 1e-40, 65504.0], dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(inputs.f32_to_bf16_bits(x), want)
    # ties: 1 + 2^-8 lies half-way between 1 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(np.float32([1.0 + 2.0 ** -8])))[0] == 1.0
    assert inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(np.float32([1.0 + 3 * 2.0 ** -8])))[0] == 1.0 + 2.0 ** -6
    back = inputs.bf16_bits_to_f32(want)
    np.testing.assert_array_equal(back, torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy())


def test_generators_are_deterministic_and_in_range():
    A1, B1, b1 = inputs.gemm_i8_case_inputs(inputs.GEMM_I8_256)
    A2, B2, b2 = inputs.gemm_i8_case_inputs(inputs.GEMM_I8_256)
    assert (A1 == A2).all() and (B1 == B2).all() and (b1 == b2).all()
    assert A1.dtype == np.int8 and A1.min() == -128 and A1.max() == 127 and b1.dtype == np.int32
    assert abs(float(A1.astype(np.float64).var()) - 5461.25) < 200
    x, w, b = inputs.conv_i8_inputs(2, 6, 6, 8, 4, 3, 3, seed=1)
    assert x.shape == (2, 6, 6, 8) and w.shape == (3, 3, 8, 4) and b.shape == (4,)
    A, B = inputs.gemm_bf16_inputs(64, 32, 48, seed=2)
    assert A.dtype == np.uint16 and A.shape == (64, 48) and B.shape == (48, 32)
    assert abs(float(inputs.bf16_bits_to_f32(A).std()) - 1.0) < 0.1
    Ab, Bb, xb, db = inputs.batched_f32_inputs(10, 12, seed=3)
    assert Ab.shape == (10, 12, 12) and xb.shape == (10, 12) and Ab.min() >= -1 and Ab.max() < 1
    seeds = [c.seed for c in inputs.GEMM_I8_SWEEP]
    assert seeds == [2000, 2001, 2002, 2003, 2004, 2005]
    assert [(c.M, c.N, c.K) for c in inputs.GEMM_I8_SWEEP][4] == (49, 2048, 4608)
