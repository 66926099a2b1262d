"""Seeded inputs for masked tree attention over a segmented KV cache: row layouts of a decoding
step (which row continues which) and random bf16 tensors.  Input generation only: nothing here
evaluates attention.

Row layout of one stream in a DS2D step (Section 3.5 of the paper): the last verified token
and the draft tokens of the tree first, level by level, then, for every one of those tokens in
the same order, its m forecast embeddings.  parent[] gives, for every row, the row it continues
(index within the stream, -1 for the last verified token): a draft token continues its parent in
the tree; forecast embedding 1 of a token continues that token, forecast embedding j > 1
continues forecast embedding j - 1 of the same token.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Sequence, Tuple

import numpy as np

from .generate import f32_to_bf16_bits


def ds2d_tree(branch: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """(parent int32 [rows], is_forecast uint8 [rows]) for a branch configuration (b_1..b_m)."""
    m = len(branch)
    parent, level = [-1], [0]
    for b in branch:
        nxt = []
        for node in level:
            for _ in range(int(b)):
                parent.append(node)
                nxt.append(len(parent) - 1)
        level = nxt
    tokens = len(parent)
    is_forecast = [0] * tokens
    for t in range(tokens):
        prev = t
        for _ in range(m):
            parent.append(prev)
            is_forecast.append(1)
            prev = len(parent) - 1
    return np.asarray(parent, np.int32), np.asarray(is_forecast, np.uint8)


def chain_tree(rows: int) -> Tuple[np.ndarray, np.ndarray]:
    """Plain autoregressive rows: each row continues the one before it."""
    return np.arange(-1, rows - 1, dtype=np.int32), np.zeros(rows, np.uint8)


def random_tree(rows: int, rng: np.random.Generator, forecast_share: float = 0.3) -> Tuple[np.ndarray, np.ndarray]:
    """Any forest-free layout: row i continues a random earlier row (row 0 is the root); rows
    marked as forecast embeddings only have forecast embeddings below them."""
    parent = np.full(rows, -1, np.int32)
    is_forecast = np.zeros(rows, np.uint8)
    for i in range(1, rows):
        parent[i] = int(rng.integers(0, i))
        is_forecast[i] = 1 if is_forecast[parent[i]] or rng.random() < forecast_share else 0
    return parent, is_forecast


@dataclass
class AttentionInputs:
    n_streams: int
    rows_per_stream: int
    scale: float
    q: np.ndarray            # uint16 [M][Hq][D]
    k_prefill: np.ndarray    # uint16 [Hkv][Lp][D]
    v_prefill: np.ndarray
    k_fprefix: np.ndarray    # uint16 [Hkv][Lf][D]
    v_fprefix: np.ndarray
    k_stream: np.ndarray     # uint16 [S][Hkv][cap][D]
    v_stream: np.ndarray
    len_stream: np.ndarray   # int32 [S]
    k_new: np.ndarray        # uint16 [M][Hkv][D]
    v_new: np.ndarray
    parent: np.ndarray       # int32 [M]
    is_forecast: np.ndarray  # uint8 [M]


def make_attention_inputs(seed: int, n_streams: int, parent: np.ndarray, is_forecast: np.ndarray,
                          Hq: int, Hkv: int, D: int, Lp: int, Lf: int, cap: int,
                          len_stream: Sequence[int] | None = None, k_std: float = 1.0) -> AttentionInputs:
    """Random tensors (q, k ~ N(0, k_std), v ~ N(0, 1), rounded to bf16) for S streams that all
    use the row layout (parent, is_forecast); stream lengths random in [0, cap] unless given."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([77, seed])))
    R = len(parent)
    M = n_streams * R

    def normal(shape, std=1.0):
        return f32_to_bf16_bits((rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).reshape(shape))

    if len_stream is None:
        len_stream = rng.integers(0, cap + 1, size=n_streams)
    return AttentionInputs(
        n_streams, R, float(1.0 / np.sqrt(D)),
        normal((M, Hq, D)), normal((Hkv, Lp, D), k_std), normal((Hkv, Lp, D)),
        normal((Hkv, Lf, D), k_std), normal((Hkv, Lf, D)),
        normal((n_streams, Hkv, cap, D), k_std), normal((n_streams, Hkv, cap, D)),
        np.asarray(len_stream, np.int32),
        normal((M, Hkv, D), k_std), normal((M, Hkv, D)),
        np.tile(np.asarray(parent, np.int32), n_streams), np.tile(np.asarray(is_forecast, np.uint8), n_streams))
