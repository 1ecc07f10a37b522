"""CPU checks of the rounding model that the attention backward's parity tests take their mean-error
tolerance from (attn_rounding_model): its unrounded branch is the oracle's definition, and its
rounded branch shows how much of the error is inherent in rounding P, dS, O and the results to bf16."""
import numpy as np
import torch

import oracle as o
from oracle import block_oracle as bo
from paper_2410_06511_amd import workloads as wl
from attn_rounding_model import mean_relative_errors, round_bf16, sdpa_bwd_with_bf16_roundings
from helpers import bits

HD = 128


def inputs(B, S, Hq, Hkv, seed, std):
    def gen(shape, seed, std):
        g = torch.Generator("cpu")
        g.manual_seed(seed)
        return o.bf16_to_f32(bits(wl.randn_bf16(shape, std, 0, generator=g))).astype(np.float64)
    qkv = gen((B * S, (Hq + 2 * Hkv) * HD), seed, std)
    return (qkv[:, :Hq * HD], qkv[:, Hq * HD:(Hq + Hkv) * HD], qkv[:, (Hq + Hkv) * HD:], gen((B * S, Hq * HD), seed + 1, 1e-2))


def test_round_bf16_is_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, -(1.0 + 2.0 ** -8 + 2.0 ** -20), 0.0])
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0, -(1.0 + 2.0 ** -7), 0.0])   # ties go to the even mantissa
    assert np.array_equal(round_bf16(x), want)
    y = np.random.default_rng(0).standard_normal(4096)
    assert np.array_equal(round_bf16(y), o.bf16_to_f32(o.f32_to_bf16(y.astype(np.float32))).astype(np.float64))


def test_unrounded_branch_is_the_definition():
    B, S, Hq, Hkv = 2, 72, 4, 2
    q, k, v, do = inputs(B, S, Hq, Hkv, 11, 1.5)
    a = sdpa_bwd_with_bf16_roundings(q, k, v, do, B, S, Hq, Hkv, HD, rounded=False)
    b = bo.sdpa_bwd_f64(q, k, v, do, B, S, Hq, Hkv, HD)
    for x, y in zip(a, b):
        assert np.abs(x - y).max() <= 1e-13 * np.abs(y).max()


def test_roundings_cost_about_one_bf16_ulp_on_average_and_three_times_that_for_peaked_scores():
    """Unit-variance inputs: 1.1 to 1.3 x 2^-9 of the mean magnitude for each gradient.  Inputs of
    standard deviation 3 (scores of order ten, softmax near one-hot): dv unchanged, dq and dk two to
    four times worse - from the roundings alone, with every sum exact."""
    flat = mean_relative_errors(*inputs(2, 200, 4, 2, 204, 1.0), 2, 200, 4, 2, HD)
    assert all(1.0 * 2.0 ** -9 <= e <= 1.3 * 2.0 ** -9 for e in flat), flat
    peaked = mean_relative_errors(*inputs(2, 264, 4, 2, 5, 3.0), 2, 264, 4, 2, HD)
    assert 2.0 * flat[0] <= peaked[0] <= 4.0 * flat[0] and 1.5 * flat[1] <= peaked[1] <= 4.0 * flat[1], (flat, peaked)
    assert 0.7 * flat[2] <= peaked[2] <= 1.3 * flat[2], (flat, peaked)
