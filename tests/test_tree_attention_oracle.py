"""Pins of the tree-attention oracle (CPU only): it is compared with things other than itself --
numpy's float64 softmax on an explicit mask built by an independent transitive closure, plain
causal attention, closed forms, invariances, and the row counts of the paper's worked example."""
import os

import numpy as np
import pytest

import oracle
import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def f64(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def run(inp, **kw):
    return oracle.tree_attention(inp.q, inp.k_prefill, inp.v_prefill, inp.k_fprefix, inp.v_fprefix,
                                 inp.k_stream, inp.v_stream, inp.len_stream, inp.k_new, inp.v_new,
                                 inp.parent, inp.is_forecast, inp.n_streams, inp.scale, **kw)


def ancestor_matrix(parent):
    """reach[i][j] = 1 if j is i or an ancestor of i: closure of the parent relation by repeated
    boolean matrix products (no pointer chasing, unlike the oracle)."""
    R = len(parent)
    step = np.eye(R, dtype=bool)
    for i, p in enumerate(parent):
        if p >= 0:
            step[i, p] = True
    reach = step.copy()
    for _ in range(R):
        reach = (reach.astype(np.int32) @ step.astype(np.int32)) > 0
    return reach


def numpy_reference(inp):
    """Dense attention with an explicit 0/1 mask over the key order prefill, forecast prefix, own
    stream segment, rows of the step; softmax via numpy in float64."""
    M, Hq, D = inp.q.shape
    Hkv, Lp = inp.k_prefill.shape[:2]
    Lf, cap = inp.k_fprefix.shape[1], inp.k_stream.shape[2]
    S, R, G = inp.n_streams, inp.rows_per_stream, Hq // Hkv
    reach = ancestor_matrix(inp.parent[:R])
    out = np.zeros((M, Hq, D))
    weights = np.zeros((M, Hq, Lp + Lf + cap + R))
    for m in range(M):
        s, i = divmod(m, R)
        for hq in range(Hq):
            hk = hq // G
            K = np.concatenate([f64(inp.k_prefill[hk]), f64(inp.k_fprefix[hk]), f64(inp.k_stream[s, hk]),
                                f64(inp.k_new[s * R:(s + 1) * R, hk])])
            V = np.concatenate([f64(inp.v_prefill[hk]), f64(inp.v_fprefix[hk]), f64(inp.v_stream[s, hk]),
                                f64(inp.v_new[s * R:(s + 1) * R, hk])])
            mask = np.concatenate([np.ones(Lp, bool), np.full(Lf, bool(inp.is_forecast[m])),
                                   np.arange(cap) < inp.len_stream[s], reach[i]])
            sc = np.where(mask, inp.scale * (K @ f64(inp.q[m, hq])), -np.inf)
            w = np.exp(sc - sc.max())
            w /= w.sum()
            weights[m, hq] = w
            out[m, hq] = w @ V
    return out, weights


@pytest.mark.parametrize("seed,tree", [(0, "ds2d"), (1, "random"), (2, "chain"), (3, "random")])
def test_matches_numpy_softmax_on_an_explicit_mask(seed, tree):
    rng = np.random.default_rng(seed)
    parent, fc = {"ds2d": wl.ds2d_tree((2, 2)), "chain": wl.chain_tree(6), "random": wl.random_tree(9, rng)}[tree]
    inp = wl.make_attention_inputs(seed, 3, parent, fc, Hq=4, Hkv=2, D=8, Lp=5, Lf=3, cap=6)
    out, w = run(inp, return_weights=True)
    ref_out, ref_w = numpy_reference(inp)
    assert np.max(np.abs(out - ref_out)) <= 1e-12 * np.max(np.abs(ref_out))
    assert np.max(np.abs(w - ref_w)) <= 1e-13
    assert np.array_equal(w == 0, ref_w == 0)                    # the same keys are invisible


def test_weights_sum_to_one_and_masked_keys_weigh_exactly_nothing():
    parent, fc = wl.ds2d_tree((3, 2))
    inp = wl.make_attention_inputs(5, 2, parent, fc, Hq=2, Hkv=1, D=16, Lp=7, Lf=4, cap=9, len_stream=[4, 0])
    out, w = run(inp, return_weights=True)
    assert np.max(np.abs(w.sum(axis=2) - 1.0)) <= 1e-14
    Lp, Lf, cap, R = 7, 4, 9, 30
    for m in range(2 * R):
        s, i = divmod(m, R)
        if not inp.is_forecast[m]:
            assert np.all(w[m, :, Lp:Lp + Lf] == 0)              # ordinary tokens never see the forecast prefix
        assert np.all(w[m, :, Lp + Lf + inp.len_stream[s]:Lp + Lf + cap] == 0)
        assert np.all(w[m, :, Lp + Lf + cap + i + 1:] == 0)      # nothing later in the step
    # poison every value a mask hides: the output must not move at all
    poisoned = wl.make_attention_inputs(5, 2, parent, fc, Hq=2, Hkv=1, D=16, Lp=7, Lf=4, cap=9, len_stream=[4, 0])
    nan = np.uint16(0x7FC0)
    poisoned.v_stream[0, :, 4:] = nan
    poisoned.v_stream[1] = nan
    poisoned.k_stream[1] = nan
    out2 = run(poisoned)
    assert np.array_equal(out, out2)


def test_worked_example_rows_see_what_the_paper_says():
    """Branch configuration (3, 2), two forecast embeddings: visible rows of the step per row."""
    path = os.path.join(ROOT, "tests", "golden", "ds2d_tree_visible_rows.txt")
    want = {int(a): int(b) for a, b in (l.split() for l in open(path) if l.strip() and not l.startswith("#"))}
    parent, fc = wl.ds2d_tree((3, 2))
    assert len(parent) == 30 and int(fc.sum()) == 20
    inp = wl.make_attention_inputs(6, 1, parent, fc, Hq=1, Hkv=1, D=8, Lp=2, Lf=1, cap=3, len_stream=[3])
    _, w = run(inp, return_weights=True)
    base = 2 + 1 + 3
    for row in range(30):
        assert int((w[row, 0, base:] > 0).sum()) == want[row], row
        assert int((w[row, 0, :2] > 0).sum()) == 2 and int((w[row, 0, 3:6] > 0).sum()) == 3
        assert (w[row, 0, 2] > 0) == bool(fc[row])


def test_identical_keys_give_the_mean_of_the_visible_values():
    """If every key is the same vector all visible weights are equal: out = mean of visible v."""
    parent, fc = wl.ds2d_tree((2, 1))
    inp = wl.make_attention_inputs(7, 2, parent, fc, Hq=2, Hkv=2, D=8, Lp=3, Lf=2, cap=4, len_stream=[1, 4])
    one = inp.k_prefill[0, 0].copy()
    for k in (inp.k_prefill, inp.k_fprefix, inp.k_stream, inp.k_new):
        k[...] = one
    out = run(inp)
    R = len(parent)
    reach = ancestor_matrix(parent)
    for m in range(2 * R):
        s, i = divmod(m, R)
        for h in range(2):
            vis = [f64(inp.v_prefill[h]), f64(inp.v_stream[s, h, :inp.len_stream[s]]),
                   f64(inp.v_new[s * R:(s + 1) * R, h][reach[i]])]
            if fc[i]:
                vis.append(f64(inp.v_fprefix[h]))
            mean = np.concatenate(vis).mean(axis=0)
            assert np.max(np.abs(out[m, h] - mean)) <= 1e-13


def test_chain_equals_plain_causal_attention():
    """Rows that each continue the previous one, no forecast rows, no prefix: ordinary causal
    attention over [prefill, stream tokens, rows so far], written here with a triangular mask."""
    parent, fc = wl.chain_tree(5)
    inp = wl.make_attention_inputs(8, 2, parent, fc, Hq=2, Hkv=1, D=8, Lp=4, Lf=0, cap=3, len_stream=[3, 2])
    out = run(inp)
    for s in range(2):
        n_ctx = 4 + int(inp.len_stream[s])
        K = np.concatenate([f64(inp.k_prefill[0]), f64(inp.k_stream[s, 0, :inp.len_stream[s]]), f64(inp.k_new[s * 5:(s + 1) * 5, 0])])
        V = np.concatenate([f64(inp.v_prefill[0]), f64(inp.v_stream[s, 0, :inp.len_stream[s]]), f64(inp.v_new[s * 5:(s + 1) * 5, 0])])
        for h in range(2):
            Q = f64(inp.q[s * 5:(s + 1) * 5, h])
            sc = inp.scale * (Q @ K.T)
            causal = np.tril(np.ones((5, 5), bool))
            sc[:, n_ctx:] = np.where(causal, sc[:, n_ctx:], -np.inf)
            p = np.exp(sc - sc.max(axis=1, keepdims=True))
            ref = (p / p.sum(axis=1, keepdims=True)) @ V
            assert np.max(np.abs(out[s * 5:(s + 1) * 5, h] - ref)) <= 1e-13


def test_streams_are_isolated_and_the_forecast_prefix_reaches_forecast_rows_only():
    parent, fc = wl.ds2d_tree((2, 2))
    R = len(parent)
    a = wl.make_attention_inputs(9, 3, parent, fc, Hq=4, Hkv=2, D=8, Lp=4, Lf=3, cap=5, len_stream=[5, 2, 3])
    out = run(a)
    # other streams' cache segments, rows and queries change: stream 1's outputs stay bit-identical
    b = wl.make_attention_inputs(10, 3, parent, fc, Hq=4, Hkv=2, D=8, Lp=4, Lf=3, cap=5, len_stream=[1, 2, 0])
    for name in ("k_prefill", "v_prefill", "k_fprefix", "v_fprefix"):
        setattr(b, name, getattr(a, name))
    for name in ("q", "k_new", "v_new"):
        getattr(b, name)[R:2 * R] = getattr(a, name)[R:2 * R]
    for name in ("k_stream", "v_stream"):
        getattr(b, name)[1] = getattr(a, name)[1]
    assert np.array_equal(run(b)[R:2 * R], out[R:2 * R])
    # a different forecast prefix moves the forecast rows and nothing else
    c = wl.make_attention_inputs(9, 3, parent, fc, Hq=4, Hkv=2, D=8, Lp=4, Lf=3, cap=5, len_stream=[5, 2, 3])
    c.v_fprefix[...] = wl.make_attention_inputs(11, 3, parent, fc, Hq=4, Hkv=2, D=8, Lp=4, Lf=3, cap=5).v_fprefix
    out_c = run(c)
    tok = np.tile(fc == 0, 3)
    assert np.array_equal(out_c[tok], out[tok])
    assert np.all(np.max(np.abs(out_c[~tok] - out[~tok]), axis=(1, 2)) > 0)


def test_query_heads_share_the_key_head_of_their_group():
    parent, fc = wl.chain_tree(3)
    inp = wl.make_attention_inputs(12, 1, parent, fc, Hq=6, Hkv=2, D=8, Lp=3, Lf=0, cap=2, len_stream=[2])
    inp.q[:, 1] = inp.q[:, 0]
    inp.q[:, 3] = inp.q[:, 0]
    out = run(inp)
    assert np.array_equal(out[:, 0], out[:, 1])                  # same group, same query -> same output
    assert np.max(np.abs(out[:, 0] - out[:, 3])) > 0             # other group: other keys and values


def test_rejects_a_parent_that_is_not_an_earlier_row():
    parent, fc = wl.chain_tree(4)
    inp = wl.make_attention_inputs(13, 2, parent, fc, Hq=1, Hkv=1, D=8, Lp=1, Lf=0, cap=1)
    inp.parent[5] = 2                                            # row 1 of stream 1 "continues" row 2
    with pytest.raises(ValueError):
        run(inp)
