"""CPU oracle for the decoder layer's glue around the int4 multi-LoRA linear: RMSNorm's per-row
scale, rotary position encoding, SwiGLU, residual.  TEST INFRASTRUCTURE ONLY: numpy in float64,
written from the definitions (the paper names these operations only as parts of its LLaMA-style
block, Section 3.1, and as targets of constant folding and operator fusion, Section 3.3 and
Table 10); shares nothing with the HIP library and is never called by it.

  rms_scale      s[m] = 1 / sqrt(mean_k x[m][k]^2 + eps)
  folding        W (g * x * s) = s * (W diag(g)) x: the norm weight g is folded into W (and into
                 the LoRA factor A) offline, which leaves the per-row scalar s at run time
  rope           heads of D features, "half-split" pairing: features (i, i + D/2) of a head are
                 rotated by angle[m][i] = position[m] * base^(-2 i / D)
  swiglu         silu(gate) * up, silu(z) = z / (1 + exp(-z)); in the fused layout every 64
                 output columns hold 32 gate columns followed by the up columns of the same features
"""
from __future__ import annotations

import numpy as np

from . import linear as _linear


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def rms_scale(x: np.ndarray, eps: float) -> np.ndarray:
    """x float64 [M][K] -> s float64 [M]."""
    x = np.asarray(x, np.float64)
    return 1.0 / np.sqrt(np.mean(x * x, axis=1) + eps)


def rope_angles(positions, head_dim: int = 64, base: float = 10000.0) -> np.ndarray:
    """angle[m][i] for i < head_dim / 2."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = base ** (-2.0 * i / head_dim)
    return np.asarray(positions, np.float64)[:, None] * inv_freq[None, :]


def rope(v: np.ndarray, cos: np.ndarray, sin: np.ndarray, head_dim: int = 64) -> np.ndarray:
    """v [M][H * head_dim]; cos, sin [M][head_dim / 2]; plain loops over heads and pairs."""
    v = np.asarray(v, np.float64)
    M, N = v.shape
    half = head_dim // 2
    out = np.empty_like(v)
    for m in range(M):
        for h in range(N // head_dim):
            for i in range(half):
                a, b = v[m, h * head_dim + i], v[m, h * head_dim + half + i]
                out[m, h * head_dim + i] = a * cos[m, i] - b * sin[m, i]
                out[m, h * head_dim + half + i] = b * cos[m, i] + a * sin[m, i]
    return out


def silu(z):
    z = np.asarray(z, np.float64)
    return z / (1.0 + np.exp(-z))


def swiglu_pairs(v: np.ndarray) -> np.ndarray:
    """Fused layout [M][N] (every 64 columns: 32 gate, 32 up) -> [M][N / 2]."""
    v = np.asarray(v, np.float64)
    M, N = v.shape
    out = np.empty((M, N // 2), np.float64)
    for t in range(N // 64):
        gate, up = v[:, 64 * t:64 * t + 32], v[:, 64 * t + 32:64 * t + 64]
        out[:, 32 * t:32 * t + 32] = silu(gate) * up
    return out


def scale_from_parts(sq_parts: np.ndarray, K: int, eps: float) -> np.ndarray:
    """Row scale of RMSNorm from partial sums of squares of a row (any partition of its K entries)."""
    return 1.0 / np.sqrt(np.sum(np.asarray(sq_parts, np.float64), axis=1) / K + eps)


def tile_squares(y: np.ndarray, tile_cols: int = 64) -> np.ndarray:
    """[M][ceil(N / tile_cols)]: sum of squares of every run of tile_cols columns of y."""
    y = np.asarray(y, np.float64)
    M, N = y.shape
    tiles = -(-N // tile_cols)
    out = np.zeros((M, tiles), np.float64)
    for t in range(tiles):
        out[:, t] = np.sum(y[:, t * tile_cols:(t + 1) * tile_cols] ** 2, axis=1)
    return out


def fused_linear(wq, scales, group, lora_a, lora_b, alpha, x_bits, row_adapter, row_scale=None,
                 pair_op: str = "none", cos=None, sin=None, residual_bits=None, sq_in=None, sq_eps: float = 0.0) -> np.ndarray:
    """The linear layer (oracle.c) followed by: row scale (given, or made from the partial sums
    of squares sq_in of the rows of x), pair operation, residual."""
    y = _linear(wq, scales, group, lora_a, lora_b, alpha, x_bits, row_adapter)
    if sq_in is not None:
        assert row_scale is None
        row_scale = scale_from_parts(sq_in, np.asarray(x_bits).shape[1], sq_eps)
    if row_scale is not None:
        y = y * np.asarray(row_scale, np.float64)[:, None]
    if pair_op == "rope":
        y = rope(y, np.asarray(cos, np.float64), np.asarray(sin, np.float64))
    elif pair_op == "swiglu":
        y = swiglu_pairs(y)
    if residual_bits is not None:
        y = y + bf16_to_f64(residual_bits)
    return y
