"""Workload shapes: the five benchmark configurations and the paper's row-count rule.

The paper runs one frozen LLaMA-style graph whose LoRA tensors are inputs
(Section 3.2, approach c), feeds it n concurrent output streams (Section 3.4)
and, per stream, a draft-token tree plus forecast embeddings (Section 3.5).
What reaches a linear layer is therefore a block of M rows with one adapter
index per row; the shapes below reproduce that structure with synthetic data.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Sequence, Tuple


@dataclass(frozen=True)
class ProjShape:
    """One projection: y[M][N] from x[M][K], int4 groups of `group` along K."""
    name: str
    K: int
    N: int
    group: int
    rank: int
    n_adapters: int
    alpha: float
    x_slot: str = "x"   # projections of a layer with the same slot share their input rows


@dataclass(frozen=True)
class Workload:
    key: str
    cfg_id: int              # first word of every seed sequence of this workload
    projs: Tuple[ProjShape, ...]
    M: int
    row_map: str             # see generate.make_rows
    layers: int
    description: str


def llama1b_layer_shapes(group: int = 32, rank: int = 16, n_adapters: int = 8,
                         alpha: float = 2.0) -> Tuple[ProjShape, ...]:
    """Seven projections of one decoder block of a 1B LLaMA-style model
    (hidden 2048, grouped K/V width 512, MLP 8192); block structure as in
    Section 3.1 of the paper, sizes from the benchmark configuration."""
    H, KV, F = 2048, 512, 8192
    mk = lambda name, K, N, slot: ProjShape(name, K, N, group, rank, n_adapters, alpha, slot)
    return (
        mk("q", H, H, "h_attn"), mk("k", H, KV, "h_attn"), mk("v", H, KV, "h_attn"),
        mk("o", H, H, "attn_out"),
        mk("gate", H, F, "h_mlp"), mk("up", H, F, "h_mlp"),
        mk("down", F, H, "mlp_act"),
    )


WORKLOADS = {
    "c1": Workload(
        "c1", 1, (ProjShape("lin", 256, 256, 32, 8, 8, 2.0),), 8, "one_to_one", 1,
        "tiny single linear, 8 streams x 1 token, row m uses adapter m"),
    "c2": Workload(
        "c2", 2, llama1b_layer_shapes(), 8, "one_to_one", 1,
        "1B-like decode step, 7 projections of one layer, 8 streams x 1 token"),
    "c3": Workload(
        "c3", 3, (ProjShape("lin", 3072, 8192, 64, 16, 8, 2.0),), 128, "block:16", 1,
        "8 streams x 16 draft-tree tokens, each stream's rows share its adapter"),
    "c3_interleaved": Workload(
        "c3_interleaved", 3, (ProjShape("lin", 3072, 8192, 64, 16, 8, 2.0),), 128,
        "interleave:8", 1, "as c3 with rows ordered node-major (m = node*8 + stream)"),
    "c4_decode": Workload(
        "c4_decode", 4, llama1b_layer_shapes(), 32, "block:4", 16,
        "16-layer stack, 8 streams x 4 tree tokens"),
    "c4_prefill": Workload(
        "c4_prefill", 4, llama1b_layer_shapes(), 512, "const:0", 16,
        "16-layer stack, prefill chunk of 512 rows from one adapter"),
    "c5_up": Workload(
        "c5_up", 5, (ProjShape("up", 4096, 14336, 128, 64, 32, 1.0),), 64, "zipf:1.1", 1,
        "skewed multi-tenant, 64 rows over 32 adapters drawn Zipf(1.1)"),
    "c5_down": Workload(
        "c5_down", 5, (ProjShape("down", 14336, 4096, 128, 64, 32, 1.0),), 64, "zipf:1.1", 1,
        "skewed multi-tenant, transposed (down) projection"),
}


def ds2d_rows(branch: Sequence[int]) -> dict:
    """Rows of one DS2D verification step for a branch configuration (b_1..b_m).

    Section 3.5: level i of the draft tree holds b_1*...*b_i tokens; the step
    verifies the D draft tokens appended to the last verified token and gives
    every one of those 1+D tokens its own m forecast embeddings.
    """
    m = len(branch)
    level, drafts = 1, 0
    for b in branch:
        level *= int(b)
        drafts += level
    tokens = 1 + drafts
    forecast = tokens * m
    return {"m": m, "draft_tokens": drafts, "tokens": tokens,
            "forecast_embeddings": forecast, "rows": tokens + forecast}


def algorithmic_bytes(p: ProjShape, M: int, n_distinct_adapters: int, y_bytes: int = 2) -> int:
    """Bytes one call has to move at least once: packed codes, fp16 scales, x, y,
    the adapters actually referenced (each once) and the row index."""
    return (p.N * p.K // 2 + 2 * p.N * (p.K // p.group) + 2 * M * p.K + y_bytes * M * p.N
            + 2 * n_distinct_adapters * p.rank * (p.K + p.N) + 4 * M)


def algorithmic_flops(p: ProjShape, M: int) -> int:
    return 2 * M * p.N * p.K + 2 * M * p.rank * (p.K + p.N)
