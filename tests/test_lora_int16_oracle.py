"""Pins of the int16-LoRA oracle (oracle/lora_int16.py): against the C oracle where int16 values
are exactly bf16 values, against a brute-force evaluation in exact rational arithmetic, against
the properties the definition fixes, and the digit identity the device-side expansion rests on."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import lora_int16 as oi
import workloads as wl


def _case(M=5, K=128, N=64, r=8, n_ad=3, seed=3):
    shape = wl.ProjShape("lin", K, N, 32, r, n_ad, 1.5)
    q = wl.make_problem_lora_int16(shape, 90, seed, 0)
    x = wl.make_x(M, K, 90, seed, 0)
    rows = np.array([(m * 2) % n_ad if m != 1 else -1 for m in range(M)], np.int32)
    return shape, q, x, rows


def test_matches_the_c_oracle_when_the_integers_are_bf16_values():
    """Small integers (|v| <= 256) are exact in bf16: with both scales 1 the definition must give
    what the C oracle gives for the same tensors handed over as bf16 (different code, different
    language: a transposed operand, a wrong index or a dropped factor shows)."""
    shape, q, x, rows = _case()
    rng = np.random.default_rng(5)
    aq = rng.integers(-256, 257, q.aq.shape).astype(np.int16)
    bq = rng.integers(-256, 257, q.bq.shape).astype(np.int16)
    a_bits = wl.f32_to_bf16_bits(aq.astype(np.float32))
    b_bits = wl.f32_to_bf16_bits(bq.astype(np.float32))
    assert np.array_equal(wl.bf16_bits_to_f32(a_bits), aq.astype(np.float32))
    want = oracle.linear(q.wq, q.scales, shape.group, a_bits, b_bits, shape.alpha, x, rows)
    got = oi.linear(q.wq, q.scales, shape.group, aq, 1.0, bq, 1.0, shape.alpha, x, rows)
    assert np.max(np.abs(got - want)) <= 1e-9 * np.max(np.abs(want))


def test_delta_against_exact_rational_arithmetic():
    M, K, N, r, n_ad = 3, 16, 5, 4, 2
    rng = np.random.default_rng(11)
    aq = rng.integers(-32767, 32768, (n_ad, r, K)).astype(np.int16)
    bq = rng.integers(-32767, 32768, (n_ad, N, r)).astype(np.int16)
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    xf = wl.bf16_bits_to_f32(x)
    rows = np.array([1, -1, 0], np.int32)
    s_a, s_b, alpha = np.float32(3.0e-5), np.float32(7.0e-6), 2.0
    got = oi.lora_delta(aq, s_a, bq, s_b, alpha, x, rows)
    for m in range(M):
        for n in range(N):
            if rows[m] < 0:
                assert got[m, n] == 0.0
                continue
            a = int(rows[m])
            acc = Fraction(0)
            for j in range(r):
                t = sum(Fraction(int(aq[a, j, k])) * Fraction(float(xf[m, k])) for k in range(K))
                acc += Fraction(int(bq[a, n, j])) * t
            want = float(Fraction(alpha) * Fraction(float(s_a)) * Fraction(float(s_b)) * acc)
            assert got[m, n] == pytest.approx(want, rel=1e-12, abs=1e-18)


def test_scales_and_alpha_are_plain_factors_and_rows_without_adapter_get_the_base():
    shape, q, x, rows = _case()
    d1 = oi.lora_delta(q.aq, q.s_a, q.bq, q.s_b, 1.0, x, rows)
    d2 = oi.lora_delta(q.aq, 2 * q.s_a, q.bq, 0.5 * q.s_b, 3.0, x, rows)
    assert np.allclose(d2, 3.0 * d1, rtol=1e-12, atol=0)
    assert np.all(d1[1] == 0.0) and np.any(d1[0] != 0.0)
    y = oi.linear(q.wq, q.scales, shape.group, q.aq, q.s_a, q.bq, q.s_b, shape.alpha, x, rows)
    none_a = np.zeros((1, 8, shape.K), np.uint16)
    none_b = np.zeros((1, shape.N, 8), np.uint16)
    base = oracle.linear(q.wq, q.scales, shape.group, none_a, none_b, 0.0, x, None)
    assert np.array_equal(y[1], base[1])


def test_quantiser_round_trip_and_range():
    rng = np.random.default_rng(2)
    t = (rng.standard_normal((3, 8, 64)) * 0.03).astype(np.float32)
    q, s = wl.quantise_lora_int16(t)
    assert q.dtype == np.int16 and np.max(np.abs(q.astype(np.int32))) == 32767
    assert np.max(np.abs(q.astype(np.float64) * float(s) - t)) <= 0.5 * float(s) * (1 + 1e-6)
    z, sz = wl.quantise_lora_int16(np.zeros((2, 8, 16), np.float32))
    assert not z.any() and sz == 1.0


def test_digit_identity_behind_the_expansion():
    """int16 = 256 hi + lo with digits that are exact in bf16; a LoRA pair of four times the rank
    built from the digits, A'' = [hi; hi; lo; lo], B'' = [65536 hi | 256 lo | 256 hi | lo], run
    through the bf16 oracle with alpha s_a s_b, is the int16 definition."""
    shape, q, x, rows = _case(M=6, K=128, N=64, r=8, n_ad=3, seed=4)
    ah, al = oi.digits(q.aq)
    bh, bl = oi.digits(q.bq)
    assert ah.min() >= -128 and ah.max() <= 127 and al.min() >= 0 and al.max() <= 255
    a4 = np.concatenate([ah, ah, al, al], axis=1).astype(np.float32)
    b4 = np.concatenate([65536 * bh, 256 * bl, 256 * bh, bl], axis=2).astype(np.float32)
    a_bits, b_bits = wl.f32_to_bf16_bits(a4), wl.f32_to_bf16_bits(b4)
    assert np.array_equal(wl.bf16_bits_to_f32(a_bits), a4) and np.array_equal(wl.bf16_bits_to_f32(b_bits), b4)
    alpha4 = float(shape.alpha) * float(q.s_a) * float(q.s_b)
    via_bf16 = oracle.linear(q.wq, q.scales, shape.group, a_bits, b_bits, alpha4, x, rows)
    want = oi.linear(q.wq, q.scales, shape.group, q.aq, q.s_a, q.bq, q.s_b, shape.alpha, x, rows)
    assert np.max(np.abs(via_bf16 - want)) <= 1e-9 * np.max(np.abs(want))
