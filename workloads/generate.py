"""Seeded generators: Gaussian weights -> packed int4 + fp16 scales, bf16 adapters and rows.

Recipe (every tensor has its own numpy PCG64 stream, seeded with
SeedSequence([cfg_id, layer, index, tensor_id])):
  w  ~ N(0, std 0.02)      -> symmetric int4 per group of G along K, fp16 scale = max|w|/7
  A  ~ N(0, variance 1/K)  -> bf16, layout [n_adapters][rank][K]
  B  ~ N(0, std 0.01)      -> bf16, layout [n_adapters][N][rank]
  x  ~ N(0, 1)             -> bf16, layout [M][K]
Encodings: bf16 and fp16 values travel as uint16 bit patterns; packed codes as
uint8 [N][K/2] with the even-k code in the low nibble, two's-complement nibbles.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

from .configs import ProjShape, Workload

T_W, T_A, T_B, T_X, T_ROWS = 0, 1, 2, 3, 4


def _rng(cfg_id: int, layer: int, index: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg_id, layer, index, tensor_id])))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """int8 codes [N][K] in [-8,7] -> uint8 [N][K/2]; even k in the low nibble."""
    c = np.ascontiguousarray(codes, dtype=np.int8).view(np.uint8) & np.uint8(0x0F)
    return (c[:, 0::2] | (c[:, 1::2] << np.uint8(4))).astype(np.uint8)


def quantise_int4(w: np.ndarray, group: int) -> Tuple[np.ndarray, np.ndarray]:
    """Symmetric group-wise int4: returns (packed uint8 [N][K/2], fp16 scale bits uint16 [N][K/group]).

    scale = fp16(max|w| / 7) over the group (1.0 if that rounds to zero),
    code = clamp(round-half-even(w / scale), -8, 7), all in float32.
    """
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, K = w.shape
    assert K % group == 0 and K % 2 == 0
    g = w.reshape(N, K // group, group)
    s32 = np.max(np.abs(g), axis=2) / np.float32(7.0)
    s16 = s32.astype(np.float16)
    s16 = np.where(s16 == 0, np.float16(1.0), s16)
    q = np.rint(g / s16.astype(np.float32)[:, :, None])
    codes = np.clip(q, -8, 7).astype(np.int8).reshape(N, K)
    return pack_nibbles(codes), s16.view(np.uint16).copy()


@dataclass
class Problem:
    """One projection's frozen tensors (host numpy arrays in the canonical layout)."""
    shape: ProjShape
    wq: np.ndarray        # uint8  [N][K/2]
    scales: np.ndarray    # uint16 [N][K/group]  (fp16 bits)
    lora_a: np.ndarray    # uint16 [n_adapters][rank][K]  (bf16 bits)
    lora_b: np.ndarray    # uint16 [n_adapters][N][rank]  (bf16 bits)


def make_problem(shape: ProjShape, cfg_id: int, layer: int, proj_index: int) -> Problem:
    p = shape
    w = _rng(cfg_id, layer, proj_index, T_W).standard_normal((p.N, p.K), dtype=np.float32)
    w *= np.float32(0.02)
    wq, scales = quantise_int4(w, p.group)
    del w
    a = _rng(cfg_id, layer, proj_index, T_A).standard_normal((p.n_adapters, p.rank, p.K), dtype=np.float32)
    a *= np.float32(1.0 / np.sqrt(p.K))
    b = _rng(cfg_id, layer, proj_index, T_B).standard_normal((p.n_adapters, p.N, p.rank), dtype=np.float32)
    b *= np.float32(0.01)
    return Problem(p, wq, scales, f32_to_bf16_bits(a), f32_to_bf16_bits(b))


def make_x(M: int, K: int, cfg_id: int, layer: int, slot_index: int) -> np.ndarray:
    x = _rng(cfg_id, layer, slot_index, T_X).standard_normal((M, K), dtype=np.float32)
    return f32_to_bf16_bits(x)


def fuse_gate_up(gate: Problem, up: Problem) -> Problem:
    """The gate and up projections of an MLP as ONE projection in the layout the fused SwiGLU
    output stage expects: every tile of 64 output rows of the weight holds 32 gate rows followed
    by the up rows of the same features (rows are quantised one by one, so codes and scales are
    just re-ordered), and the two LoRA pairs become one of twice the rank:
    A = [A_gate; A_up], B = [[B_gate, 0], [0, B_up]] re-ordered like the weight rows."""
    g, u = gate.shape, up.shape
    assert (g.K, g.N, g.group, g.rank, g.n_adapters, g.alpha) == (u.K, u.N, u.group, u.rank, u.n_adapters, u.alpha)
    assert g.N % 32 == 0
    F, r, n_ad = g.N, g.rank, g.n_adapters
    order = np.empty(2 * F, np.int64)                      # fused row -> row of concat(gate, up)
    for t in range(F // 32):
        order[64 * t:64 * t + 32] = np.arange(32 * t, 32 * t + 32)
        order[64 * t + 32:64 * t + 64] = F + np.arange(32 * t, 32 * t + 32)
    wq = np.concatenate([gate.wq, up.wq], axis=0)[order]
    scales = np.concatenate([gate.scales, up.scales], axis=0)[order]
    lora_a = np.concatenate([gate.lora_a, up.lora_a], axis=1)              # [n_ad][2r][K]
    b = np.zeros((n_ad, 2 * F, 2 * r), np.uint16)
    b[:, :F, :r] = gate.lora_b
    b[:, F:, r:] = up.lora_b
    shape = ProjShape("gate_up", g.K, 2 * F, g.group, 2 * r, n_ad, g.alpha)
    return Problem(shape, np.ascontiguousarray(wq), np.ascontiguousarray(scales), np.ascontiguousarray(lora_a),
                   np.ascontiguousarray(b[:, order, :]))


def quantise_act_int8(x: np.ndarray) -> Tuple[np.ndarray, np.float32]:
    """Per-tensor symmetric int8 quantisation of activations (Section 3.3 of the paper): one
    scale max|x| / 127 in float32 (1 for an all-zero tensor), round to nearest even, clamp."""
    x = np.asarray(x, np.float32)
    top = np.float32(np.max(np.abs(x))) if x.size else np.float32(0)
    scale = np.float32(top / np.float32(127.0)) if top > 0 else np.float32(1.0)
    q = np.clip(np.rint(x / scale), -127, 127).astype(np.int8)
    return q, scale


def make_x_int8(M: int, K: int, cfg_id: int, layer: int, slot_index: int) -> Tuple[np.ndarray, np.float32]:
    """The same N(0, 1) rows as make_x, quantised to int8 with one scale for the tensor."""
    x = _rng(cfg_id, layer, slot_index, T_X).standard_normal((M, K), dtype=np.float32)
    return quantise_act_int8(x)


def quantise_lora_int16(t: np.ndarray) -> Tuple[np.ndarray, np.float32]:
    """Symmetric int16 quantisation of a stack of LoRA tensors with ONE scale for the stack:
    s = max|t| / 32767 in float32 (1 for an all-zero stack), round to nearest even, clamp."""
    t = np.asarray(t, np.float32)
    top = np.float32(np.max(np.abs(t))) if t.size else np.float32(0)
    scale = np.float32(top / np.float32(32767.0)) if top > 0 else np.float32(1.0)
    q = np.clip(np.rint(t / scale), -32767, 32767).astype(np.int16)
    return q, scale


@dataclass
class ProblemLoraInt16:
    """A projection whose LoRA tensors are int16 with one scale per stack (the base weight as in Problem)."""
    shape: ProjShape
    wq: np.ndarray        # uint8  [N][K/2]
    scales: np.ndarray    # uint16 [N][K/group]  (fp16 bits)
    aq: np.ndarray        # int16 [n_adapters][rank][K]
    s_a: np.float32
    bq: np.ndarray        # int16 [n_adapters][N][rank]
    s_b: np.float32


def make_problem_lora_int16(shape: ProjShape, cfg_id: int, layer: int, proj_index: int) -> ProblemLoraInt16:
    """The tensors of make_problem with the LoRA stacks quantised to int16 instead of rounded to bf16."""
    p = shape
    w = _rng(cfg_id, layer, proj_index, T_W).standard_normal((p.N, p.K), dtype=np.float32)
    w *= np.float32(0.02)
    wq, scales = quantise_int4(w, p.group)
    del w
    a = _rng(cfg_id, layer, proj_index, T_A).standard_normal((p.n_adapters, p.rank, p.K), dtype=np.float32)
    a *= np.float32(1.0 / np.sqrt(p.K))
    b = _rng(cfg_id, layer, proj_index, T_B).standard_normal((p.n_adapters, p.N, p.rank), dtype=np.float32)
    b *= np.float32(0.01)
    aq, s_a = quantise_lora_int16(a)
    bq, s_b = quantise_lora_int16(b)
    return ProblemLoraInt16(p, wq, scales, aq, s_a, bq, s_b)


def make_rows(row_map: str, M: int, n_adapters: int, cfg_id: int = 0) -> np.ndarray:
    """Row -> adapter index (int32 [M]).

    one_to_one     a(m) = m mod n_adapters          (streams x 1 token)
    block:B        a(m) = (m div B) mod n_adapters  (stream-major rows, B tree tokens per stream)
    interleave:S   a(m) = m mod S                   (node-major rows, S streams)
    const:c        a(m) = c                         (one adapter per call, the paper's own case)
    zipf:s         a(m) drawn with p(k) ~ (k+1)^-s  (skewed multi-tenant)
    """
    kind, _, arg = row_map.partition(":")
    m = np.arange(M)
    if kind == "one_to_one":
        a = m % n_adapters
    elif kind == "block":
        a = (m // int(arg)) % n_adapters
    elif kind == "interleave":
        a = m % int(arg)
    elif kind == "const":
        a = np.full(M, int(arg))
    elif kind == "zipf":
        p = (np.arange(n_adapters) + 1.0) ** (-float(arg))
        p /= p.sum()
        a = _rng(cfg_id, 0, 0, T_ROWS).choice(n_adapters, size=M, p=p)
    else:
        raise ValueError(f"unknown row map {row_map!r}")
    return a.astype(np.int32)


def make_layer_inputs(wl: Workload, layer: int = 0) -> Tuple[None, List[np.ndarray], np.ndarray]:
    """The rows of one layer of a workload without its weights: (None, xs, row_adapter), the
    same xs and rows that make_layer returns."""
    slots: Dict[Tuple[str, int], np.ndarray] = {}
    xs = []
    for s in wl.projs:
        key = (s.x_slot, s.K)
        if key not in slots:
            slots[key] = make_x(wl.M, s.K, wl.cfg_id, layer, len(slots))
        xs.append(slots[key])
    rows = make_rows(wl.row_map, wl.M, wl.projs[0].n_adapters, wl.cfg_id)
    return None, xs, rows


def make_layer(wl: Workload, layer: int = 0) -> Tuple[List[Problem], List[np.ndarray], np.ndarray]:
    """All projections of one layer of a workload: (problems, xs, row_adapter).

    xs[i] is the input of projection i; projections naming the same x_slot get
    the very same array object (q/k/v and gate/up share their rows).
    """
    problems = [make_problem(s, wl.cfg_id, layer, i) for i, s in enumerate(wl.projs)]
    _, xs, rows = make_layer_inputs(wl, layer)
    return problems, xs, rows
