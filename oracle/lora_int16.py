"""CPU oracle for LoRA tensors stored as int16 with one scale per tensor.  TEST INFRASTRUCTURE ONLY.

The paper's deployment keeps the LoRA weights in 16-bit integers (appendix on the 1B model: the
memory comparison's paragraph names int16 LoRA weights next to int4 base weights).  It does not
say how the scale is chosen; the reading taken here is symmetric quantisation with ONE scale for
the stack of A tensors of a projection and one for its B tensors:

    A[a] ~ s_a * Aq[a],   B[a] ~ s_b * Bq[a]          Aq, Bq int16

so that the linear of Section 3.1 (Eq. 1-4) becomes

    y[m] = dequant(Wq, scales) x[m] + alpha * s_a * s_b * Bq[a(m)] (Aq[a(m)] x[m]).

Everything below is the definition written out in float64 with numpy (integers up to 2^15 times
bf16 values: every product is exact in float64, sums are float64 sums).  The base term comes from
the C oracle's linear() called without adapters.
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64: the 16 bits are the top half of a float32."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def lora_delta(aq, s_a, bq, s_b, alpha, x_bits, row_adapter):
    """alpha * s_a * s_b * Bq[a(m)] (Aq[a(m)] x[m]) for every row, float64 [M][N]; rows whose
    adapter index is negative get zeros.  aq int16 [n][r][K], bq int16 [n][N][r], x bf16 bits [M][K]."""
    aq = np.asarray(aq)
    bq = np.asarray(bq)
    assert aq.dtype == np.int16 and bq.dtype == np.int16
    n, r, K = aq.shape
    N = bq.shape[1]
    assert bq.shape == (n, N, r)
    x = bf16_bits_to_f64(x_bits)
    M = x.shape[0]
    assert x.shape == (M, K) and len(row_adapter) == M
    out = np.zeros((M, N), np.float64)
    for m in range(M):
        a = int(row_adapter[m])
        if a < 0:
            continue
        if a >= n:
            raise ValueError("row_adapter index outside [-1, n_adapters)")
        t = float(s_a) * (aq[a].astype(np.float64) @ x[m])               # [r]   (shrink, Eq. 2)
        out[m] = float(alpha) * float(s_b) * (bq[a].astype(np.float64) @ t)   # [N]   (expand, Eq. 3)
    return out


def linear(wq, scales, group, aq, s_a, bq, s_b, alpha, x_bits, row_adapter):
    """y [M][N] float64: base product of the C oracle (no adapters) + lora_delta."""
    import oracle
    K = wq.shape[1] * 2
    N = wq.shape[0]
    none_a = np.zeros((1, 8, K), np.uint16)
    none_b = np.zeros((1, N, 8), np.uint16)
    base = oracle.linear(wq, scales, group, none_a, none_b, 0.0, x_bits, None)
    return base + lora_delta(aq, s_a, bq, s_b, alpha, x_bits, row_adapter)


def digits(v: np.ndarray):
    """The two base-256 digits of int16 values: v = 256 * hi + lo with hi in [-128, 127] and lo in
    [0, 255] (floor division), both int32."""
    v = np.asarray(v).astype(np.int32)
    hi = v >> 8
    lo = v & 255
    assert np.array_equal(256 * hi + lo, v)
    return hi, lo
