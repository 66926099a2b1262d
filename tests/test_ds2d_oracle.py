"""Pins of the DS2D step oracle (oracle/ds2d.py) against things other than itself: the counts of
the paper's worked example, the defining property of speculative decoding (the tokens given out
equal plain greedy decoding of the same model, whatever the drafts), library sorting, and an
independently written tree layout.  Mutated steps must fail the same checks."""
import itertools
import os

import numpy as np
import pytest

from oracle import ds2d
from workloads.attention import ds2d_tree

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden_counts():
    """The counts the paper states for its worked example, and the branch configurations of its
    Table 7 (tests/golden/ds2d_worked_example.txt)."""
    out, table7 = {}, []
    for line in open(os.path.join(GOLDEN, "ds2d_worked_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, value = line.split()
        vals = [int(v) for v in value.split(",")]
        if key == "table7":
            table7.append(tuple(vals))
        else:
            out[key] = vals
    return out, table7


def test_worked_example_counts():
    g, table7 = golden_counts()
    m, branch = g["m"][0], g["branch"]
    parent, is_forecast, level = ds2d.tree_rows(branch, m)
    n_tok = ds2d.n_tokens(branch)
    assert n_tok == g["tokens"][0]
    assert n_tok - 1 == g["draft_tokens"][0]
    assert int(is_forecast.sum()) == g["forecast_embeddings"][0]
    assert len(parent) == g["rows"][0]
    assert int(((level == 1) & (is_forecast == 0)).sum()) == branch[0]
    # the first step has no drafts: the last prompt token and its forecast embeddings
    p1, f1, _ = ds2d.tree_rows((), m)
    assert list(p1) == [-1, 0, 1] and list(f1) == [0, 1, 1]
    # every configuration of Table 7 fits the row budget the paper fixes
    for cfg in table7:
        rows = len(ds2d.tree_rows(cfg, len(cfg))[0])
        assert rows == ds2d.n_tokens(cfg) * (1 + len(cfg)) <= g["row_budget"][0]


def test_tree_rows_against_the_input_generators_layout_and_the_hand_written_depths():
    for branch in [(3, 2), (2, 2, 2), (1,), (4,), (2, 1, 3), (1, 1, 1, 1)]:
        parent, is_forecast, level = ds2d.tree_rows(branch, len(branch))
        p2, f2 = ds2d_tree(branch)
        assert np.array_equal(parent, p2) and np.array_equal(is_forecast, f2)
    # rows visible within the step = length of the chain to the root (file written by hand)
    parent, _, _ = ds2d.tree_rows((3, 2), 2)
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(GOLDEN, "ds2d_tree_visible_rows.txt"))
            if l.strip() and not l.startswith("#")]
    for row, visible in rows:
        n, a = 0, row
        while a >= 0:
            n, a = n + 1, parent[a]
        assert n == visible
    # fewer levels than forecast embeddings, and none at all
    parent, is_forecast, level = ds2d.tree_rows((2,), 3)
    assert len(parent) == 3 * 4 and list(parent[:3]) == [-1, 0, 0]
    assert list(parent[3:6]) == [0, 3, 4] and list(level[3:6]) == [1, 2, 3]


def test_best_tokens_against_numpy_sorting():
    rng = np.random.default_rng(5)
    v = rng.standard_normal(500)
    assert ds2d.best_tokens(v, 7) == list(np.argsort(-v, kind="stable")[:7])
    # ties: lower id first; -0 equals +0; NaN last, -inf before NaN
    v = np.array([1.0, 3.0, 3.0, -0.0, 0.0, np.nan, -np.inf, 3.0])
    assert ds2d.best_tokens(v, 8) == [1, 2, 7, 0, 3, 4, 6, 5]
    assert ds2d.best_tokens(np.array([np.nan, np.nan]), 1) == [0]
    # brute force on tiny inputs: all orderings of a multiset
    for perm in itertools.permutations([2.0, 2.0, 1.0, -1.0]):
        got = ds2d.best_tokens(np.array(perm), 3)
        want = sorted(range(4), key=lambda i: (-perm[i], i))[:3]
        assert got == want


# ---------------------------------------------------------------- the defining property
V = 40


def model_logits(context):
    """A deterministic toy language model: logits depend on the whole token sequence."""
    seed = 1469598103934665603
    for t in context:
        seed = ((seed ^ (int(t) + 1)) * 1099511628211) % (1 << 64)
    return np.random.default_rng(seed).standard_normal(V)


def greedy(prompt, n):
    seq = list(prompt)
    for _ in range(n):
        seq.append(int(np.argmax(model_logits(seq))))
    return seq[len(prompt):]


def forecast_logits(context, j, quality, rng, rank):
    """Logits of forecast embedding j after `context` (which ends with the token the embedding is
    attached to): with probability `quality` the token plain decoding would produce j + 1 places
    later sits at position `rank` of the ordering, otherwise the row is noise."""
    row = rng.standard_normal(V)
    if rng.random() < quality:
        truth = greedy(context, j + 1)[-1]
        order = np.argsort(-row, kind="stable")
        row[truth] = (row[order[rank]] + (row[order[rank - 1]] if rank else row[order[0]] + 2.0)) / 2 \
            if truth not in order[:rank] else row[truth]
    return row


def decode(step_fn, prompt, branch, m, quality, n_steps, seed):
    """Run DS2D steps with the toy model; returns (tokens given out, per-step counts)."""
    rng = np.random.default_rng(seed)
    verified = list(prompt)                    # ends with the last verified token
    cur_branch, tokens = (), [prompt[-1]]
    out, counts = [], []
    for _ in range(n_steps):
        parent, is_forecast, level = ds2d.tree_rows(cur_branch, m)
        n_tok = ds2d.n_tokens(cur_branch)
        paths = []
        for r in range(n_tok):
            chain, a = [], r
            while a > 0:
                chain.append(tokens[a])
                a = parent[a]
            paths.append(verified + chain[::-1])
        logits = np.zeros((len(parent), V))
        for r in range(n_tok):
            logits[r] = model_logits(paths[r])
            for j in range(1, m + 1):
                rank = int(rng.integers(0, branch[j - 1]))
                logits[n_tok + r * m + j - 1] = forecast_logits(paths[r], j, quality, rng, rank)
        res = step_fn(cur_branch, branch, m, logits, tokens)
        # what was given out continues the verified text
        verified += res["emitted"]
        out += res["emitted"]
        counts.append(len(res["emitted"]))
        assert res["next_tokens"][0] == res["emitted"][-1]
        cur_branch, tokens = tuple(branch), list(res["next_tokens"])
    return out, counts


@pytest.mark.parametrize("branch", [(3, 2), (2, 2, 2), (4,), (1, 1)])
@pytest.mark.parametrize("quality", [0.0, 0.6, 1.0])
def test_tokens_given_out_equal_plain_greedy_decoding(branch, quality):
    m = len(branch)
    prompt = [3, 17, 5]
    out, counts = decode(ds2d.step, prompt, branch, m, quality, 6, seed=11)
    assert out == greedy(prompt, len(out))
    assert counts[0] == 1                       # the first step has nothing to verify
    if quality == 1.0:
        assert all(c == 1 + m for c in counts[1:])      # every level accepted, every step
    if quality == 0.0:
        assert sum(counts) < 6 * (1 + m)


def test_new_drafts_come_from_the_node_where_the_walk_ended_and_from_nowhere_else():
    g, _ = golden_counts()
    m, branch = g["m"][0], tuple(g["branch"])
    rng = np.random.default_rng(3)
    n_tok = ds2d.n_tokens(branch)
    logits = rng.standard_normal((n_tok * (1 + m), V))
    tokens = [9] + [int(t) for t in rng.integers(0, V, n_tok - 1)]
    # accept root -> second first-level draft (row 2) -> its first child (row 6)
    tokens[1], tokens[2], tokens[3] = 1, 2, 3
    logits[0, 2] = 50.0
    tokens[6], tokens[7] = 20, 21
    logits[2, 20] = 50.0
    res = ds2d.step(branch, branch, m, logits, tokens)
    # (the paper's figure has three tokens accepted in a row -- the root, a first-level and a
    # second-level draft -- and the new drafts taken from the last of them)
    assert res["accepted_rows"] == [0, 2, 6]
    assert res["emitted"][:2] == [2, 20] and res["emitted"][2] == int(np.argmax(logits[6]))
    rows = [n_tok + 6 * m, n_tok + 6 * m + 1]
    top1 = list(np.argsort(-logits[rows[0]], kind="stable")[:3])
    top2 = list(np.argsort(-logits[rows[1]], kind="stable")[:2])
    assert res["next_tokens"] == [res["emitted"][2]] + top1 + top2 * 3
    # other forecast rows do not matter; these two do
    other = logits.copy()
    for r in range(n_tok, logits.shape[0]):
        if r not in rows:
            other[r] = rng.standard_normal(V)
    assert ds2d.step(branch, branch, m, other, tokens) == res
    other = logits.copy()
    other[rows[1], (top2[0] + 1) % V] = 99.0
    assert ds2d.step(branch, branch, m, other, tokens)["next_tokens"] != res["next_tokens"]


# ---------------------------------------------------------------- planted mistakes must be caught
def _no_bonus(cb, nb, m, logits, tokens):
    r = ds2d.step(cb, nb, m, logits, tokens)
    if len(r["emitted"]) > 1:
        r = dict(r, emitted=r["emitted"][:-1], next_tokens=[r["emitted"][-2]] + r["next_tokens"][1:])
    return r


def _accept_first_child(cb, nb, m, logits, tokens):
    r = ds2d.step(cb, nb, m, logits, tokens)
    if len(cb) and len(r["accepted_rows"]) == 1:           # accepts a draft that was not confirmed
        r = dict(r, emitted=[int(tokens[1])] + r["emitted"])
    return r


def _forecast_rows_of_the_root(cb, nb, m, logits, tokens):
    r = ds2d.step(cb, nb, m, logits, tokens)
    n_tok = ds2d.n_tokens(cb)
    nt, width = [r["next_tokens"][0]], 1
    for i, b in enumerate(nb, start=1):
        cand = ds2d.best_tokens(logits[n_tok + i - 1], b)          # always the root's embeddings
        width *= b
        nt += [cand[q % b] for q in range(width)]
    return dict(r, next_tokens=nt)


def _levels_swapped(cb, nb, m, logits, tokens):
    r = ds2d.step(cb, nb, m, logits, tokens)
    n_tok = ds2d.n_tokens(cb)
    cur = r["accepted_rows"][-1]
    nt, width = [r["next_tokens"][0]], 1
    for i, b in enumerate(nb, start=1):
        cand = ds2d.best_tokens(logits[n_tok + cur * m + (m - i)], b)   # embedding m + 1 - i for level i
        width *= b
        nt += [cand[q % b] for q in range(width)]
    return dict(r, next_tokens=nt)


@pytest.mark.parametrize("mutant", [_no_bonus, _accept_first_child, _forecast_rows_of_the_root, _levels_swapped])
def test_planted_mistakes_fail_the_property(mutant):
    branch, m, prompt = (3, 2), 2, [3, 17, 5]
    failed = False
    for quality in (1.0, 0.5):
        try:
            out, counts = decode(mutant, prompt, branch, m, quality, 8, seed=11)
            failed |= out != greedy(prompt, len(out))
            failed |= quality == 1.0 and not all(c == 1 + m for c in counts[1:])
        except AssertionError:
            failed = True
    assert failed, mutant.__name__
