"""Seeded inputs for the DS2D step: logits of all rows of a step and the token ids at its token
rows.  Input generation only: nothing here verifies or drafts.

Logits are rounded to bf16 when asked (as a bf16 language-model head produces them), which makes
equal values common, so the order among equals matters.  To make drafts get accepted, a spike is
planted, with probability `accept`, in a token row's logits at the token id carried by one of the
rows that continue it."""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np

from .generate import f32_to_bf16_bits


def make_ds2d_inputs(seed: int, n_streams: int, branch: Sequence[int], m: int, vocab: int, bf16: bool,
                     accept: float = 0.6, std: float = 2.0) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (logits, tokens): logits [S * R][V] as uint16 bf16 patterns or float32, tokens
    int32 [S][T].  The tree has len(branch) levels and m forecast embeddings per token."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([91, seed])))
    # token rows of the tree: level by level, the children of one node next to each other
    parent = [-1]
    frontier = [0]
    for b in branch:
        grown = []
        for node in frontier:
            for _ in range(int(b)):
                parent.append(node)
                grown.append(len(parent) - 1)
        frontier = grown
    T = len(parent)
    R = T * (1 + m)
    logits = (rng.standard_normal((n_streams * R, vocab), dtype=np.float32) * np.float32(std))
    tokens = rng.integers(0, vocab, size=(n_streams, T)).astype(np.int32)
    for s in range(n_streams):
        for node in range(T):
            kids = [c for c in range(T) if parent[c] == node]
            if kids:
                # distinct tokens among the children of a node, as a top-b choice produces them
                tokens[s, kids] = rng.choice(vocab, size=len(kids), replace=False).astype(np.int32)
                if rng.random() < accept:
                    logits[s * R + node, tokens[s, kids[int(rng.integers(0, len(kids)))]]] = np.float32(40.0)
    if bf16:
        return f32_to_bf16_bits(logits), tokens
    return logits, tokens
