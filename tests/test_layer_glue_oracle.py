"""Pins of oracle/layer_glue.py against things other than itself: complex-number rotations and
the relative-position property of rotary encodings, scipy's logistic function, direct numpy
formulas, and the folding identity of RMSNorm's weight."""
import numpy as np
import pytest
from scipy.special import expit

import oracle
import workloads as wl
from oracle import layer_glue as glue
from workloads.generate import bf16_bits_to_f32, f32_to_bf16_bits


def test_rms_scale_against_the_direct_formula_and_known_rows():
    x = np.array([[3.0, 4.0, 0.0, 0.0], [1.0, 1.0, 1.0, 1.0], [0.0, 0.0, 0.0, 0.0]])
    s = glue.rms_scale(x, 0.0 + 1e-6)
    assert np.allclose(s[0], 1.0 / np.sqrt(25.0 / 4 + 1e-6), rtol=1e-15)
    assert np.allclose(s[1], 1.0 / np.sqrt(1.0 + 1e-6), rtol=1e-15)
    assert np.allclose(s[2], 1000.0, rtol=1e-12)             # eps alone
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64))
    y = x * glue.rms_scale(x, 0.0)[:, None]
    assert np.allclose(np.mean(y * y, axis=1), 1.0, rtol=1e-13)   # normalised rows have unit mean square


def test_norm_weight_folds_into_the_weight_matrix():
    """W (g * x * s) == s * (W diag(g)) x: what is left at run time is the scalar per row."""
    rng = np.random.default_rng(1)
    W, g, x = rng.standard_normal((7, 32)), rng.standard_normal(32), rng.standard_normal((3, 32))
    s = glue.rms_scale(x, 1e-5)
    lhs = (x * s[:, None] * g[None, :]) @ W.T
    rhs = s[:, None] * (x @ (W * g[None, :]).T)
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-12)


def test_rope_is_a_complex_rotation_and_depends_on_relative_position_only():
    rng = np.random.default_rng(2)
    M, H = 6, 3
    v = rng.standard_normal((M, H * 64))
    pos = np.array([0, 1, 5, 17, 100, 2048])
    ang = glue.rope_angles(pos)
    out = glue.rope(v, np.cos(ang), np.sin(ang))
    # complex view: feature pair (i, i + 32) of a head is re + j im, multiplied by exp(j angle)
    z = (v.reshape(M, H, 2, 32)[:, :, 0] + 1j * v.reshape(M, H, 2, 32)[:, :, 1]) * np.exp(1j * ang)[:, None, :]
    want = np.stack([z.real, z.imag], axis=2).reshape(M, H * 64)
    assert np.allclose(out, want, rtol=1e-13, atol=1e-13)
    assert np.array_equal(out[0], v[0])                            # position 0: identity
    assert np.allclose(np.linalg.norm(out, axis=1), np.linalg.norm(v, axis=1), rtol=1e-13)
    # first frequency is 1 radian per position, the last one base^(-62/64)
    assert np.isclose(ang[1, 0], 1.0) and np.isclose(ang[1, 31], 10000.0 ** (-62.0 / 64))
    # <rope(q, p), rope(k, p')> depends on p - p' only
    q, k = rng.standard_normal((1, 64)), rng.standard_normal((1, 64))
    def dot(p, p2):
        a, b = glue.rope_angles([p]), glue.rope_angles([p2])
        return float((glue.rope(q, np.cos(a), np.sin(a)) @ glue.rope(k, np.cos(b), np.sin(b)).T)[0, 0])
    assert np.isclose(dot(7, 3), dot(104, 100), rtol=1e-10) and not np.isclose(dot(7, 3), dot(7, 4))


def test_silu_and_the_fused_gate_up_layout():
    z = np.array([-30.0, -1.0, 0.0, 1.0, 30.0])
    assert np.allclose(glue.silu(z), z * expit(z), rtol=1e-14, atol=1e-300)
    assert glue.silu(0.0) == 0.0 and np.isclose(glue.silu(30.0), 30.0, rtol=1e-12)
    rng = np.random.default_rng(3)
    gate, up = rng.standard_normal((4, 96)), rng.standard_normal((4, 96))
    fused = np.empty((4, 192))
    for t in range(3):
        fused[:, 64 * t:64 * t + 32] = gate[:, 32 * t:32 * t + 32]
        fused[:, 64 * t + 32:64 * t + 64] = up[:, 32 * t:32 * t + 32]
    assert np.allclose(glue.swiglu_pairs(fused), gate * expit(gate) * up, rtol=1e-14)


def test_fused_gate_up_projection_equals_two_separate_projections():
    """One weight whose tiles hold 32 gate rows then 32 up rows, with a LoRA pair of twice the
    rank (block-diagonal B): the fused oracle must equal silu(gate(x)) * up(x) from two plain
    oracle calls on the original tensors."""
    K, F, r, n_ad, M = 128, 64, 8, 2, 5
    pg = wl.make_problem(wl.ProjShape("gate", K, F, 32, r, n_ad, 2.0), 801, 0, 0)
    pu = wl.make_problem(wl.ProjShape("up", K, F, 32, r, n_ad, 2.0), 801, 0, 1)
    x = wl.make_x(M, K, 801, 0, 0)
    rows = np.array([0, 1, -1, 1, 0], np.int32)
    fused = wl.fuse_gate_up(pg, pu)
    got = glue.fused_linear(fused.wq, fused.scales, 32, fused.lora_a, fused.lora_b, 2.0, x, rows, pair_op="swiglu")
    g = oracle.linear(pg.wq, pg.scales, 32, pg.lora_a, pg.lora_b, 2.0, x, rows)
    u = oracle.linear(pu.wq, pu.scales, 32, pu.lora_a, pu.lora_b, 2.0, x, rows)
    assert np.allclose(got, g * expit(g) * u, rtol=1e-12, atol=1e-12)


def test_fused_linear_order_of_operations():
    p = wl.make_problem(wl.ProjShape("q", 128, 64, 32, 8, 2, 2.0), 802, 0, 0)
    x = wl.make_x(3, 128, 802, 0, 0)
    rows = np.array([1, -1, 0], np.int32)
    y = oracle.linear(p.wq, p.scales, 32, p.lora_a, p.lora_b, 2.0, x, rows)
    s = np.array([0.5, 2.0, 3.0])
    ang = glue.rope_angles([3, 9, 4])
    res = f32_to_bf16_bits(np.full((3, 64), 0.25, np.float32))
    got = glue.fused_linear(p.wq, p.scales, 32, p.lora_a, p.lora_b, 2.0, x, rows, s, "rope", np.cos(ang), np.sin(ang), res)
    want = glue.rope(y * s[:, None], np.cos(ang), np.sin(ang)) + 0.25
    assert np.allclose(got, want, rtol=1e-13)
    # the scale commutes with the rotation, the residual does not
    assert not np.allclose(got, glue.rope(y * s[:, None] + 0.25, np.cos(ang), np.sin(ang)))


def test_scale_from_partial_sums_of_squares_equals_the_direct_scale():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((6, 200))
    parts = glue.tile_squares(x)                                   # runs of 64 columns, the last one short
    assert parts.shape == (6, 4) and np.isclose(parts[2, 3], np.sum(x[2, 192:] ** 2))
    assert np.allclose(glue.scale_from_parts(parts, 200, 1e-5), glue.rms_scale(x, 1e-5), rtol=1e-14)
    # any partition of a row gives the same scale
    other = np.stack([np.sum(x[:, :7] ** 2, axis=1), np.sum(x[:, 7:] ** 2, axis=1)], axis=1)
    assert np.allclose(glue.scale_from_parts(other, 200, 1e-5), glue.rms_scale(x, 1e-5), rtol=1e-14)
