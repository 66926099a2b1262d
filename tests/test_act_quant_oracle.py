"""Pins of the int8-activation oracle (oracle/act_quant.c) against things other than itself: the
already pinned bf16 oracle on exactly representable activations, numpy integer products, and the
quantiser's rounding and range rules."""
import numpy as np
import pytest

import oracle
import workloads as wl
from workloads.generate import bf16_bits_to_f32, f32_to_bf16_bits


def problem(seed, K=256, N=96, G=32, r=8, n_ad=3):
    return wl.make_problem(wl.ProjShape("t", K, N, G, r, n_ad, 2.0), 700 + seed, 0, 0)


@pytest.mark.parametrize("G", [32, 64, 128])
@pytest.mark.parametrize("exp", [-6, 0, 3])
def test_equals_the_bf16_oracle_when_the_scale_is_a_power_of_two(G, exp):
    """s_x = 2^exp: s_x * xq has at most 7 significant bits, so it is exact in bf16 and the layer
    on int8 activations must be the plain layer on those bf16 rows."""
    p = problem(G + exp, K=256, N=80, G=G, r=16, n_ad=3)
    rng = np.random.default_rng(G * 10 + exp + 100)
    xq = rng.integers(-127, 128, size=(9, 256)).astype(np.int8)
    rows = np.array([0, 2, -1, 1, 1, 0, -1, 2, 2], np.int32)
    s_x = float(2.0 ** exp)
    x_bits = f32_to_bf16_bits((xq.astype(np.float32) * np.float32(s_x)))
    assert np.array_equal(bf16_bits_to_f32(x_bits), xq.astype(np.float32) * np.float32(s_x))
    ref = oracle.linear(p.wq, p.scales, G, p.lora_a, p.lora_b, 2.0, x_bits, rows)
    got = oracle.linear_a8(p.wq, p.scales, G, p.lora_a, p.lora_b, 2.0, xq, s_x, rows)
    assert np.max(np.abs(got - ref)) <= 1e-12 * np.max(np.abs(ref))
    # and without adapters
    ref0 = oracle.linear(p.wq, p.scales, G, p.lora_a, p.lora_b, 2.0, x_bits, None)
    got0 = oracle.linear_a8(p.wq, p.scales, G, p.lora_a, p.lora_b, 2.0, xq, s_x, None)
    assert np.max(np.abs(got0 - ref0)) <= 1e-12 * np.max(np.abs(ref0))
    assert np.max(np.abs(got - got0)) > 0


def test_unit_scales_give_numpy_integer_products_times_the_activation_scale():
    p = problem(1, K=128, N=64, G=32, r=8, n_ad=1)
    codes = oracle.unpack_codes(p.wq).astype(np.int64)            # [N][K]
    ones = np.full(p.scales.shape, 0x3C00, np.uint16)             # fp16 1.0
    rng = np.random.default_rng(2)
    xq = rng.integers(-127, 128, size=(5, 128)).astype(np.int8)
    got = oracle.linear_a8(p.wq, ones, 32, p.lora_a, p.lora_b, 2.0, xq, 0.375, None)
    want = (xq.astype(np.int64) @ codes.T).astype(np.float64) * 0.375
    assert np.array_equal(got, want)
    # extreme values on both sides: |sum| = 128 inputs x 8 x 127
    wq_min = np.full_like(p.wq, 0x88)                             # every code -8
    xmax = np.full((1, 128), 127, np.int8)
    got = oracle.linear_a8(wq_min, ones, 32, p.lora_a, p.lora_b, 2.0, xmax, 1.0, None)
    assert np.all(got == -8 * 127 * 128)


def test_scale_is_linear_and_group_scales_are_taken_per_group():
    p = problem(3, K=256, N=48, G=64, r=8, n_ad=2)
    rng = np.random.default_rng(3)
    xq = rng.integers(-127, 128, size=(4, 256)).astype(np.int8)
    rows = np.array([1, 0, -1, 1], np.int32)
    y1 = oracle.linear_a8(p.wq, p.scales, 64, p.lora_a, p.lora_b, 2.0, xq, 0.01, rows)
    y3 = oracle.linear_a8(p.wq, p.scales, 64, p.lora_a, p.lora_b, 2.0, xq, 0.03, rows)
    assert np.allclose(y3, 3 * y1, rtol=1e-13)
    # activations that are non-zero in one group only see that group's scale
    only = np.zeros((1, 256), np.int8)
    only[0, 128:192] = xq[0, 128:192]
    w = oracle.dequant(p.wq, p.scales, 64)                        # [N][K] float64
    want = (w[:, 128:192] @ only[0, 128:192].astype(np.float64)) * 0.5
    got = oracle.linear_a8(p.wq, p.scales, 64, p.lora_a, p.lora_b, 2.0, only, 0.5, None)[0]
    assert np.allclose(got, want, rtol=1e-13)


def test_quantiser_rounding_range_and_agreement_with_the_generators():
    x = np.array([127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 63.49, -127.0, 0.0], np.float32)
    xq, s = oracle.quantise_act(x)
    assert s == np.float32(1.0)
    assert list(xq) == [127, 0, 2, 2, 0, -2, -2, 63, -127, 0]      # ties to even
    xq, s = oracle.quantise_act(np.zeros(7, np.float32))
    assert s == np.float32(1.0) and not xq.any()
    rng = np.random.default_rng(5)
    for _ in range(5):
        x = (rng.standard_normal((6, 300)) * rng.uniform(0.01, 50)).astype(np.float32)
        xq, s = oracle.quantise_act(x)
        assert s == np.float32(np.max(np.abs(x))) / np.float32(127)
        assert np.max(np.abs(xq.astype(np.int32))) == 127
        assert np.max(np.abs(x - s * xq.astype(np.float32))) <= 0.5 * s * (1 + 1e-6)
        q2, s2 = wl.quantise_act_int8(x)
        assert s2 == s and np.array_equal(q2, xq)
