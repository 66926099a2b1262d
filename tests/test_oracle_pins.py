"""Pins for the CPU oracle: each test checks it against something other than itself
(closed forms, integer-exact cases, numpy's float64 matmul, brute force on tiny
shapes, hand-written fixtures), chosen so that a dropped term, a wrong sign or
index, or a transposed operand fails at least one of them.  CPU only.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ONE_F16 = 0x3C00
ONE_BF16 = 0x3F80


def bf16_exact(values):
    """bf16 bit patterns of values that are exactly representable (small integers, halves)."""
    v = np.asarray(values, np.float32)
    bits = wl.f32_to_bf16_bits(v)
    assert np.array_equal(wl.bf16_bits_to_f32(bits), v)
    return bits


def small_problem(seed, K=64, N=24, G=32, r=4, n_ad=3, M=5):
    rng = np.random.default_rng(seed)
    codes = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    wq = wl.pack_nibbles(codes)
    scales = rng.uniform(0.001, 0.02, size=(N, K // G)).astype(np.float16).view(np.uint16)
    A = wl.f32_to_bf16_bits(rng.standard_normal((n_ad, r, K)).astype(np.float32) / np.sqrt(K))
    B = wl.f32_to_bf16_bits(rng.standard_normal((n_ad, N, r)).astype(np.float32) * 0.01)
    x = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    rows = rng.integers(-1, n_ad, size=M).astype(np.int32)
    return dict(codes=codes, wq=wq, scales=scales, G=G, A=A, B=B, x=x, rows=rows)


def as_f64(bits16, kind):
    if kind == "bf16":
        return wl.bf16_bits_to_f32(bits16).astype(np.float64)
    return np.asarray(bits16, np.uint16).view(np.float16).astype(np.float64)


# ---------------------------------------------------------------- 16-bit float widening

def test_f16_and_bf16_widening_against_numpy_all_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref16 = bits.view(np.float16).astype(np.float64)
    with np.errstate(invalid="ignore"):
        ref_bf = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    for b in range(65536):                # every bit pattern of both formats
        got = oracle.f16_to_double(b)
        assert (np.isnan(got) and np.isnan(ref16[b])) or got == ref16[b]
        got = oracle.bf16_to_double(b)
        assert (np.isnan(got) and np.isnan(ref_bf[b])) or got == ref_bf[b]


def test_f32_to_f16_rounding_against_numpy():
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.standard_normal(2000).astype(np.float32) * np.float32(0.01),
        rng.standard_normal(500).astype(np.float32) * np.float32(1e-6),      # subnormal range
        np.array([0.0, 1.0, 65504.0, 65519.9, 65520.0, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25,
                  0.00048828125 * (1 + 2 ** -11), 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11,
                  2047.5 / 1024, 6.1e-5], np.float32)])
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    for v, r in zip(vals, ref):
        assert oracle.f32_to_f16(float(v)) == int(r), v


# ---------------------------------------------------------------- unpack

def test_unpack_hand_written_bytes():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "nibble_bytes.txt"))
            if l.strip() and not l.startswith("#")]
    wq = np.array([[int(r[0], 16) for r in rows]], np.uint8)
    expect = np.array([[c for r in rows for c in (int(r[1]), int(r[2]))]], np.int8)
    assert np.array_equal(oracle.unpack_codes(wq), expect)


def test_unpack_every_code_in_every_nibble_position():
    # all 256 byte values: low nibble -> even k, high nibble -> odd k
    wq = np.arange(256, dtype=np.uint8).reshape(4, 64)
    codes = oracle.unpack_codes(wq)
    signed = lambda nib: nib - 16 if nib >= 8 else nib
    for n in range(4):
        for j in range(64):
            byte = n * 64 + j
            assert codes[n, 2 * j] == signed(byte & 15)
            assert codes[n, 2 * j + 1] == signed(byte >> 4)


def test_pack_unpack_round_trip_and_generator_packer_agree():
    rng = np.random.default_rng(2)
    codes = rng.integers(-8, 8, size=(37, 96)).astype(np.int8)
    wq = oracle.pack_codes(codes)
    assert np.array_equal(oracle.unpack_codes(wq), codes)
    assert np.array_equal(wl.pack_nibbles(codes), wq)


def test_dequant_is_code_times_scale_exactly():
    p = small_problem(3)
    w = oracle.dequant(p["wq"], p["scales"], p["G"])
    s = as_f64(p["scales"], "f16")
    expect = p["codes"].astype(np.float64) * np.repeat(s, p["G"], axis=1)
    assert np.array_equal(w, expect)


# ---------------------------------------------------------------- quantiser (makes the inputs)

def test_quantiser_invariants_and_agreement_with_generator():
    rng = np.random.default_rng(4)
    w = (rng.standard_normal((48, 256)) * 0.02).astype(np.float32)
    w[5, 32:64] = 0.0                                  # an all-zero group
    for G in (32, 64, 128):
        wq_o, s_o = oracle.quantise(w, G)
        wq_g, s_g = wl.quantise_int4(w, G)
        assert np.array_equal(wq_o, wq_g) and np.array_equal(s_o, s_g)
        codes = oracle.unpack_codes(wq_o).reshape(48, 256 // G, G)
        s = as_f64(s_o, "f16")
        wg = w.astype(np.float64).reshape(48, 256 // G, G)
        nonzero = np.abs(wg).max(axis=2) > 0
        assert np.all(np.abs(codes).max(axis=2)[nonzero] == 7)
        assert np.all(codes[~nonzero] == 0) and np.all(s[~nonzero] == 1.0)
        # scale is max/7 rounded to fp16: within half an fp16 ulp (2^-11 relative)
        assert np.all(np.abs(s[nonzero] - np.abs(wg).max(axis=2)[nonzero] / 7)
                      <= s[nonzero] * 2.0 ** -11)
        # reconstruction error at most half a step (plus the float32 division's rounding)
        err = np.abs(wg - codes * s[:, :, None])
        assert np.all(err <= 0.5 * s[:, :, None] * (1 + 1e-6))


# ---------------------------------------------------------------- base term

def test_base_ones_input_closed_form():
    # x = 1 everywhere: y[n] = sum_g scale[n][g] * (integer sum of the group's codes)
    p = small_problem(5, K=128, N=16, G=32, M=2)
    x = np.full((2, 128), ONE_BF16, np.uint16)
    y = oracle.linear(p["wq"], p["scales"], 32, p["A"], p["B"], 2.0, x, np.full(2, -1, np.int32))
    for n in range(16):
        total = Fraction(0)
        for g in range(4):
            isum = int(p["codes"][n, 32 * g:32 * g + 32].astype(np.int64).sum())
            total += Fraction(float(as_f64(p["scales"][n, g], "f16"))) * isum
        assert abs(y[0, n] - float(total)) <= 1e-15 * max(1.0, abs(float(total)))
        assert y[1, n] == y[0, n]


def test_base_integer_exact():
    # scales = 1, small-integer x: every product and sum is an exact integer
    rng = np.random.default_rng(6)
    codes = rng.integers(-8, 8, size=(20, 64)).astype(np.int8)
    xi = rng.integers(-4, 5, size=(7, 64))
    y = oracle.linear(wl.pack_nibbles(codes), np.full((20, 2), ONE_F16, np.uint16), 32,
                      np.zeros((1, 4, 64), np.uint16), np.zeros((1, 20, 4), np.uint16), 1.0,
                      bf16_exact(xi), np.full(7, -1, np.int32))
    assert np.array_equal(y, (xi.astype(np.int64) @ codes.astype(np.int64).T).astype(np.float64))


def test_base_single_nonzero_weight_picks_the_right_x_and_scale():
    # one code, one scale group, one x column: catches transposed / shifted indexing
    N, K, G, M = 6, 128, 32, 3
    for (n0, k0) in [(0, 0), (5, 127), (2, 33), (3, 64)]:
        codes = np.zeros((N, K), np.int8)
        codes[n0, k0] = -5
        scales = np.full((N, K // G), ONE_F16, np.uint16)
        scales[n0, k0 // G] = np.float16(0.25).view(np.uint16)
        scales[(n0 + 1) % N, k0 // G] = np.float16(8.0).view(np.uint16)      # decoys
        scales[n0, (k0 // G + 1) % (K // G)] = np.float16(16.0).view(np.uint16)
        xv = np.arange(M * K, dtype=np.float32).reshape(M, K) % 97 - 48       # exact in bf16
        y = oracle.linear(wl.pack_nibbles(codes), scales, G, np.zeros((1, 4, K), np.uint16),
                          np.zeros((1, N, 4), np.uint16), 1.0, bf16_exact(xv),
                          np.full(M, -1, np.int32))
        expect = np.zeros((M, N))
        expect[:, n0] = -5 * 0.25 * xv[:, k0]
        assert np.array_equal(y, expect)


def test_base_matches_numpy_matmul_on_dequantised_matrix():
    p = small_problem(7, K=256, N=40, G=64, M=9)
    y = oracle.linear(p["wq"], p["scales"], 64, p["A"], p["B"], 2.0, p["x"],
                      np.full(9, -1, np.int32))
    w = p["codes"].astype(np.float64) * np.repeat(as_f64(p["scales"], "f16"), 64, axis=1)
    ref = as_f64(p["x"], "bf16") @ w.T
    assert np.max(np.abs(y - ref)) <= 1e-12 * np.max(np.abs(ref))


# ---------------------------------------------------------------- LoRA term

def test_zero_B_and_no_adapter_reproduce_base_exactly():
    p = small_problem(8)
    base = oracle.linear(p["wq"], p["scales"], p["G"], p["A"], p["B"], 2.0, p["x"],
                         np.full(5, -1, np.int32))
    zero_b = oracle.linear(p["wq"], p["scales"], p["G"], p["A"], np.zeros_like(p["B"]), 2.0,
                           p["x"], np.array([0, 1, 2, 0, 1], np.int32))
    none_rows = oracle.linear(p["wq"], p["scales"], p["G"], p["A"], p["B"], 2.0, p["x"], None)
    assert np.array_equal(base, zero_b) and np.array_equal(base, none_rows)


def test_merged_weight_brute_force():
    # Eq. 1-4: XW + X(sAB) = X(W + sAB); merged matrix built with numpy per adapter
    p = small_problem(9, K=64, N=12, G=32, r=4, n_ad=3, M=6)
    rows = np.array([2, 0, 1, 1, -1, 2], np.int32)
    alpha = 1.75
    y, t = oracle.linear(p["wq"], p["scales"], 32, p["A"], p["B"], alpha, p["x"], rows,
                         return_t=True)
    w = p["codes"].astype(np.float64) * np.repeat(as_f64(p["scales"], "f16"), 32, axis=1)
    A, B, x = as_f64(p["A"], "bf16"), as_f64(p["B"], "bf16"), as_f64(p["x"], "bf16")
    for m, a in enumerate(rows):
        merged = w if a < 0 else w + alpha * (B[a] @ A[a])          # [N][K]
        ref = merged @ x[m]
        assert np.max(np.abs(y[m] - ref)) <= 1e-12 * np.max(np.abs(ref))
        t_ref = np.zeros(4) if a < 0 else A[a] @ x[m]
        assert np.max(np.abs(t[m] - t_ref)) <= 1e-13 * max(1.0, np.max(np.abs(t_ref)))


def test_rank_one_closed_form_and_alpha_is_a_direct_multiplier():
    # zero base weight, rank 1: y[m][n] = alpha * b[n] * (a . x[m]); exact with small integers
    K, N, M = 32, 5, 3
    a_vec = (np.arange(K) % 5 - 2).astype(np.float32)
    b_vec = np.array([1, -2, 3, 0, 4], np.float32)
    xv = (np.arange(M * K).reshape(M, K) % 7 - 3).astype(np.float32)
    A = bf16_exact(a_vec.reshape(1, 1, K))
    B = bf16_exact(b_vec.reshape(1, N, 1))
    for alpha in (1.0, 2.0, 0.5):
        y = oracle.linear(np.zeros((N, K // 2), np.uint8), np.full((N, 1), ONE_F16, np.uint16),
                          32, A, B, alpha, bf16_exact(xv), np.zeros(M, np.int32))
        expect = alpha * np.outer(xv.astype(np.float64) @ a_vec.astype(np.float64), b_vec)
        assert np.array_equal(y, expect)


def test_lora_index_layouts_single_nonzero_entries():
    # one nonzero A entry and one nonzero B entry: only (adapter, j, k) and (adapter, n, j)
    # read in the stated layouts [n_adapters][rank][K], [n_adapters][N][rank] give the result
    K, N, r, n_ad, M = 64, 7, 4, 3, 4
    A = np.zeros((n_ad, r, K), np.float32)
    B = np.zeros((n_ad, N, r), np.float32)
    A[1, 2, 37] = 3.0
    B[1, 5, 2] = -2.0
    B[1, 5, 3] = 64.0      # decoy: t[., 3] is zero
    B[2, 5, 2] = 32.0      # decoy: other adapter
    xv = (np.arange(M * K).reshape(M, K) % 11 - 5).astype(np.float32)
    rows = np.array([1, 2, 1, 0], np.int32)
    y = oracle.linear(np.zeros((N, K // 2), np.uint8), np.full((N, 2), ONE_F16, np.uint16), 32,
                      bf16_exact(A), bf16_exact(B), 2.0, bf16_exact(xv), rows)
    expect = np.zeros((M, N))
    for m in (0, 2):
        expect[m, 5] = 2.0 * -2.0 * 3.0 * xv[m, 37]
    assert np.array_equal(y, expect)


def test_one_hot_mask_over_all_adapters_equals_indexed_adapter():
    # Section 3.2: approach (b) (all LoRAs resident, one-hot mask) selects what approach (c) feeds
    p = small_problem(10, n_ad=4, M=6)
    rows = np.array([3, 0, 2, 2, 1, 0], np.int32)
    y = oracle.linear(p["wq"], p["scales"], p["G"], p["A"], p["B"], 2.0, p["x"], rows)
    base = oracle.linear(p["wq"], p["scales"], p["G"], p["A"], p["B"], 2.0, p["x"], None)
    A, B, x = as_f64(p["A"], "bf16"), as_f64(p["B"], "bf16"), as_f64(p["x"], "bf16")
    for m, a in enumerate(rows):
        masked = sum((1.0 if i == a else 0.0) * (B[i] @ (A[i] @ x[m])) for i in range(4))
        ref = base[m] + 2.0 * masked
        assert np.max(np.abs(y[m] - ref)) <= 1e-12 * np.max(np.abs(ref))


# ---------------------------------------------------------------- batching

def test_rows_are_independent_and_permutation_equivariant():
    p = small_problem(11, M=7)
    y = oracle.linear(p["wq"], p["scales"], p["G"], p["A"], p["B"], 2.0, p["x"], p["rows"])
    for m in range(7):                                   # streams are independent (Section 3.4)
        y1 = oracle.linear(p["wq"], p["scales"], p["G"], p["A"], p["B"], 2.0,
                           p["x"][m:m + 1], p["rows"][m:m + 1])
        assert np.array_equal(y1[0], y[m])
    perm = np.random.default_rng(0).permutation(7)
    yp = oracle.linear(p["wq"], p["scales"], p["G"], p["A"], p["B"], 2.0,
                       p["x"][perm], p["rows"][perm])
    assert np.array_equal(yp, y[perm])


def test_linearity_in_x():
    p = small_problem(12, M=4)
    xa = (np.random.default_rng(1).integers(-8, 9, size=(4, 64))).astype(np.float32)
    xb = (np.random.default_rng(2).integers(-8, 9, size=(4, 64))).astype(np.float32)
    rows = np.array([0, 1, 2, 1], np.int32)
    f = lambda xv: oracle.linear(p["wq"], p["scales"], p["G"], p["A"], p["B"], 2.0,
                                 bf16_exact(xv), rows)
    lhs, rhs = f(xa + 2 * xb), f(xa) + 2 * f(xb)
    assert np.max(np.abs(lhs - rhs)) <= 1e-12 * np.max(np.abs(lhs))


def test_thread_count_does_not_change_results():
    p = small_problem(13, N=64, M=6)
    oracle.set_threads(1)
    y1 = oracle.linear(p["wq"], p["scales"], p["G"], p["A"], p["B"], 2.0, p["x"], p["rows"])
    oracle.set_threads(4)
    y4 = oracle.linear(p["wq"], p["scales"], p["G"], p["A"], p["B"], 2.0, p["x"], p["rows"])
    assert np.array_equal(y1, y4)


# ---------------------------------------------------------------- grouping

def check_grouping(rows, n_ad):
    perm, seg_adapter, seg_start = oracle.group_rows(rows, n_ad)
    M = len(rows)
    with_adapter = sorted((m for m in range(M) if rows[m] >= 0), key=lambda m: (rows[m], m))
    without = [m for m in range(M) if rows[m] < 0]
    assert list(perm) == with_adapter + without
    assert sorted(perm) == list(range(M))
    assert list(seg_adapter) == sorted(set(int(a) for a in rows if a >= 0))
    assert seg_start[0] == 0 if len(seg_start) else True
    assert seg_start[-1] == len(with_adapter)
    for s, a in enumerate(seg_adapter):
        seg = perm[seg_start[s]:seg_start[s + 1]]
        assert len(seg) > 0 and all(rows[m] == a for m in seg)
        assert list(seg) == sorted(seg)


def test_group_rows_brute_force():
    rng = np.random.default_rng(14)
    for M, n_ad in [(1, 1), (8, 8), (128, 8), (64, 32), (257, 5), (33, 64)]:
        check_grouping(rng.integers(-1, n_ad, size=M).astype(np.int32), n_ad)
    check_grouping(np.full(16, -1, np.int32), 4)
    check_grouping(np.zeros(0, np.int32), 4)
    check_grouping(np.full(40, 3, np.int32), 4)
    for key in ("c1", "c3", "c3_interleaved", "c4_decode", "c4_prefill", "c5_up"):
        w = wl.WORKLOADS[key]
        check_grouping(wl.make_rows(w.row_map, w.M, w.projs[0].n_adapters, w.cfg_id),
                       w.projs[0].n_adapters)


def test_group_rows_every_assignment_of_a_tiny_case():
    for rows in itertools.product(range(-1, 3), repeat=4):
        check_grouping(np.array(rows, np.int32), 3)


def test_group_rows_rejects_out_of_range():
    with pytest.raises(ValueError):
        oracle.group_rows(np.array([0, 4], np.int32), 4)
    with pytest.raises(ValueError):
        oracle.group_rows(np.array([-2, 0], np.int32), 4)


# ---------------------------------------------------------------- DS2D row arithmetic

def test_ds2d_rows_worked_example_and_table7_budget():
    facts, table7 = {}, []
    for line in open(os.path.join(GOLDEN, "ds2d_worked_example.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        key, value = line.split()
        if key == "table7":
            table7.append(tuple(int(v) for v in value.split(",")))
        else:
            facts[key] = value
    got = wl.ds2d_rows(tuple(int(v) for v in facts["branch"].split(",")))
    for key in ("m", "draft_tokens", "tokens", "forecast_embeddings", "rows"):
        assert got[key] == int(facts[key]), key
    budget = int(facts["row_budget"])
    assert len(table7) == 9
    for branch in table7:
        assert wl.ds2d_rows(branch)["rows"] <= budget, branch
