"""GPU parity of mlora_ds2d_step (through the C ABI) against oracle/ds2d.py: every output is an
integer and must match exactly."""
import numpy as np
import pytest

from oracle import ds2d as oracle_ds2d
from workloads.ds2d import make_ds2d_inputs
from workloads.generate import bf16_bits_to_f32

pytestmark = pytest.mark.gpu


def run_step(gpu, S, m, branch, next_branch, V, logits, tokens, bf16):
    lib, device, torch = gpu
    d = lib.Ds2dStep(S, m, branch, next_branch, V, lib.Y_BF16 if bf16 else lib.Y_FP32)
    T_next, _ = lib.ds2d_rows(next_branch, m)
    lg = torch.from_numpy(logits.view(np.int16) if bf16 else logits).cuda()
    tk = torch.from_numpy(np.ascontiguousarray(tokens, np.int32)).cuda()
    n_acc = torch.full((S,), -7, dtype=torch.int32, device="cuda")
    rows = torch.full((S, m + 1), -7, dtype=torch.int32, device="cuda")
    emitted = torch.full((S, m + 1), -7, dtype=torch.int32, device="cuda")
    nxt = torch.full((S, T_next), -7, dtype=torch.int32, device="cuda")
    ws = torch.empty(max(16, d.workspace_bytes()), dtype=torch.uint8, device="cuda")
    ws.fill_(0xAB)                                # scratch needs no initialisation
    d.run(lg, tk, n_acc, rows, emitted, nxt, ws)
    torch.cuda.synchronize()
    return n_acc.cpu().numpy(), rows.cpu().numpy(), emitted.cpu().numpy(), nxt.cpu().numpy()


def check(gpu, S, m, branch, next_branch, V, logits, tokens, bf16):
    values = bf16_bits_to_f32(logits).astype(np.float64) if bf16 else logits.astype(np.float64)
    T, R = oracle_ds2d.n_tokens(branch), oracle_ds2d.n_tokens(branch) * (1 + m)
    n_acc, rows, emitted, nxt = run_step(gpu, S, m, branch, next_branch, V, logits, tokens, bf16)
    lengths = []
    for s in range(S):
        ref = oracle_ds2d.step(branch, next_branch, m, values[s * R:(s + 1) * R], tokens[s])
        a = len(ref["accepted_rows"]) - 1
        lengths.append(a)
        assert n_acc[s] == a
        assert list(rows[s]) == ref["accepted_rows"] + [-1] * (m - a)
        assert list(emitted[s]) == ref["emitted"] + [-1] * (m - a)
        assert list(nxt[s]) == ref["next_tokens"]
    return lengths


@pytest.mark.parametrize("S,m,branch,next_branch,V,bf16", [
    (2, 2, (3, 2), (3, 2), 1000, True),            # the paper's worked example, two streams
    (1, 2, (3, 2), (3, 2), 128256, True),          # a large vocabulary: 32 slices per row
    (3, 2, (3, 2), (2, 2), 5003, False),           # fp32 logits, rows not 16-byte aligned
    (3, 2, (3, 2), (3, 2), 5003, True),            # bf16 rows at odd element offsets
    (4, 2, (), (3, 2), 777, True),                 # the first step: nothing to verify
    (2, 3, (2, 2, 2), (2, 2, 2), 4097, True),      # one logit in the second slice
    (2, 3, (2, 2), (1, 3), 3, False),              # tiny vocabulary, next tree needs all of it
    (5, 1, (15,), (15,), 300, True),               # widest level
    (2, 4, (1, 1, 1, 1), (1, 1, 1, 1), 64, False),  # a chain
    (3, 2, (3, 2), (), 900, True),                 # the next step drafts nothing
    (40, 2, (3, 2), (3, 2), 2048, True),           # many streams
])
def test_ds2d_step_matches_oracle(gpu, S, m, branch, next_branch, V, bf16):
    seen = set()
    for seed in range(3):
        logits, tokens = make_ds2d_inputs(seed, S, branch, m, V, bf16, accept=0.7)
        seen |= set(check(gpu, S, m, branch, next_branch, V, logits, tokens, bf16))
    if len(branch) >= 2 and S * 3 >= 9 and V > 100:
        assert len(seen) >= 2, seen                 # walks of different lengths occurred


def test_ds2d_ties_signed_zeros_nan_and_infinities(gpu):
    S, m, branch, V = 3, 2, (3, 2), 600
    T, R = 10, 30
    rng = np.random.default_rng(4)
    logits = np.zeros((S * R, V), np.float32)                    # stream 0: everything equal
    logits[R:2 * R] = rng.choice(np.array([0.0, -0.0, 1.0, -1.0], np.float32), size=(R, V))
    weird = rng.standard_normal((R, V)).astype(np.float32)
    weird[rng.random((R, V)) < 0.3] = np.nan
    weird[rng.random((R, V)) < 0.1] = -np.inf
    weird[rng.random((R, V)) < 0.02] = np.inf
    weird[3] = np.nan                                            # a row of NaN only
    weird[T + 2] = -np.inf
    logits[2 * R:] = weird
    tokens = np.zeros((S, T), np.int32)
    tokens[:, 1:] = rng.integers(0, 4, size=(S, T - 1))
    tokens[0, 1:4] = [2, 0, 1]                                   # all-equal logits: arg-max is token 0
    tokens[0, 6:8] = [5, 0]                                      # children of row 2: accept row 7
    check(gpu, S, m, branch, branch, V, logits, tokens, False)
    n_acc, rows, _, _ = run_step(gpu, S, m, branch, branch, V, logits, tokens, False)
    assert n_acc[0] == 2 and list(rows[0]) == [0, 2, 7]


def test_ds2d_tokens_outside_the_vocabulary_never_match(gpu):
    S, m, branch, V = 1, 2, (3, 2), 500
    logits, tokens = make_ds2d_inputs(9, S, branch, m, V, True, accept=0.0)
    tokens[0, 1:] = [-1, V, 2 ** 31 - 1, -5, V + 3, 7 * V, -2, -3, -4]
    assert check(gpu, S, m, branch, branch, V, logits, tokens, True) == [0]


def test_ds2d_branch_configurations_of_table_7(gpu):
    """Every branch configuration the paper lists in Table 7 (read from the golden file that
    also pins their row counts), each followed by each other as the next step's tree."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "ds2d_worked_example.txt")
    table7 = [tuple(int(v) for v in l.split()[1].split(",")) for l in open(path) if l.startswith("table7")]
    assert len(table7) == 9
    by_m = {}
    for cfg in table7:
        by_m.setdefault(len(cfg), []).append(cfg)
    for m, cfgs in by_m.items():
        for i, cur in enumerate(cfgs):
            nxt = cfgs[(i + 1) % len(cfgs)]
            logits, tokens = make_ds2d_inputs(20 + i, 3, cur, m, 1531, True, accept=0.8)
            check(gpu, 3, m, cur, nxt, 1531, logits, tokens, True)
