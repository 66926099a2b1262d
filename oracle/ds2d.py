"""CPU oracle for one DS2D decoding step: verification of the draft tree and drafting of the
next one.  TEST INFRASTRUCTURE ONLY: plain Python and numpy, written from the paper's
description (Section 3.5, Appendix A.2); shares nothing with the HIP library and is never
called by it.

The step, per output stream.  The model has m forecast embeddings.  The rows of the step are
the tokens of a tree (the last verified token as root, then the draft tokens level by level:
level i has b_1 * ... * b_i nodes, the children of one node next to each other) followed, for
every token in the same order, by its m forecast embeddings.  The forward pass has produced one
row of logits per row of the step.

 1. Verification (greedy).  Start at the root.  The token the model itself continues a node with
    is the arg-max of that node's logits.  If one of the node's children carries exactly that
    token, the child is accepted and the walk goes on from it; otherwise, or at a leaf, the walk
    ends.  The tokens given out by the step are those of the accepted drafts followed by the
    arg-max at the node where the walk ended (the next "last verified token").
 2. Drafting.  The forecast embeddings of the node where the walk ended predict what follows
    that next token: level i of the new tree is filled from the b_i highest logits of forecast
    embedding i, best first, the same b_i tokens below every node of level i - 1.

The paper speaks of sampling after a soft-max; here both choices are the deterministic ones
(highest logit first, which is also highest probability first).  Order of candidates: larger
logit first; equal logits (+0 and -0 are equal), lower token id first; NaN after everything else.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np


def tree_rows(branch: Sequence[int], m: int):
    """Row tables of one stream for a tree with the given branch tuple (may be shorter than m,
    or empty: the first step has no drafts) and m forecast embeddings per token.
    Returns (parent, is_forecast, level): parent = row continued (-1 at the root); level = depth
    of a token in the tree, and for a forecast embedding its number 1..m."""
    parent, level = [-1], [0]
    frontier = [0]
    for depth, b in enumerate(branch, start=1):
        grown = []
        for node in frontier:
            for _ in range(int(b)):
                parent.append(node)
                level.append(depth)
                grown.append(len(parent) - 1)
        frontier = grown
    n_tok = len(parent)
    is_forecast = [0] * n_tok
    for tok in range(n_tok):
        for j in range(1, m + 1):
            parent.append(tok if j == 1 else len(parent) - 1)
            level.append(j)
            is_forecast.append(1)
    return np.asarray(parent, np.int32), np.asarray(is_forecast, np.uint8), np.asarray(level, np.int32)


def n_tokens(branch: Sequence[int]) -> int:
    total, width = 1, 1
    for b in branch:
        width *= int(b)
        total += width
    return total


def best_tokens(logits_row: np.ndarray, k: int) -> List[int]:
    """The k best token ids of one row of logits in the order stated at the top."""
    v = np.asarray(logits_row, np.float64)
    order = sorted(range(v.shape[0]), key=lambda i: (1, 0.0, i) if np.isnan(v[i]) else (0, -v[i], i))
    return order[:k]


def step(cur_branch: Sequence[int], next_branch: Sequence[int], m: int, logits: np.ndarray,
         tokens: Sequence[int]) -> Dict[str, object]:
    """One stream.  logits [rows][V] of the current step, tokens [n_tok] the token ids at its
    token rows.  Returns accepted_rows (root first), emitted (accepted draft tokens, then the
    next last verified token), next_tokens (token rows of the next step for next_branch)."""
    parent, is_forecast, _ = tree_rows(cur_branch, m)
    n_tok = n_tokens(cur_branch)
    assert logits.shape[0] == len(parent) and len(tokens) == n_tok and len(next_branch) <= m
    cur, path = 0, [0]
    while True:
        target = best_tokens(logits[cur], 1)[0]
        nxt = [c for c in range(n_tok) if parent[c] == cur and int(tokens[c]) == target]
        if not nxt:
            break
        cur = nxt[0]
        path.append(cur)
    emitted = [int(tokens[r]) for r in path[1:]] + [target]
    next_tokens = [target]
    width = 1
    for i, b in enumerate(next_branch, start=1):
        forecast_row = n_tok + cur * m + (i - 1)
        assert is_forecast[forecast_row]
        cand = best_tokens(logits[forecast_row], int(b))
        width *= int(b)
        next_tokens += [cand[q % int(b)] for q in range(width)]
    return {"accepted_rows": path, "emitted": emitted, "next_tokens": next_tokens}
