"""One decoder layer of a LLaMA-style model as a sequence of library calls (Section 3.1 of the
paper: attention and MLP blocks with LoRA on every projection), with the glue folded into the
projections' output stages:

    s1 = rms_scale(h)                                   mlora_rms_scale (first layer of a stack only)
    q, k, v = fused(h; row scale s1; RoPE on q and k)   mlora_w4_layer_step_fused, one launch
    attn = tree_attention(q, cache, k, v)               mlora_tree_attention, two launches
    h2 = fused(attn; + residual h; leaves the sums     o projection
         of squares of the rows of h2, per column tile)
    act = fused(h2; row scale from those sums; SwiGLU)  gate and up as one projection
    out = fused(act; + residual h2; leaves the sums     down projection
          of squares of its rows for the next layer)

The first normalisation takes its row scale from mlora_rms_scale unless the caller hands in the
sums of squares the previous layer's down projection left (h_sq): a stack of layers then needs
the rms kernel for its first layer only.

Argument marshalling only: every step runs in the library's kernels.  The norm weights are
folded into the projections offline, the gate and up weights are stored as one projection with
interleaved tiles (see include/mlora_w4.h)."""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B


class DecoderLayerStep:
    def __init__(self, proj_q, proj_k, proj_v, proj_o, proj_gate_up, proj_down, attention: B.TreeAttention,
                 h, rope_cos, rope_sin, row_adapter, M: int, eps: float = 1e-5, h_sq=None):
        """proj_*: binding.Proj on the device; attention: descriptor whose k_new / v_new are the
        tensors this step writes k and v to; h bf16 [M][hidden] (int16 tensor); rope tables fp32
        [M][32]."""
        dev = h.device
        hidden, ffn = proj_q.K, proj_gate_up.N // 2
        i16 = lambda n: torch.empty((M, n), dtype=torch.int16, device=dev)
        self.M, self.eps, self.h, self.attention = M, eps, h, attention
        parts = (hidden + 63) // 64                      # column tiles of a projection that writes hidden columns
        self.s1 = torch.empty(M, dtype=torch.float32, device=dev)
        self.h_sq = h_sq                                 # [M][parts] from the previous layer, or None
        self.sq2 = torch.empty((M, parts), dtype=torch.float32, device=dev)
        self.out_sq = torch.empty((M, parts), dtype=torch.float32, device=dev)
        self.q = i16(proj_q.N)
        self.k_new, self.v_new = attention.keep[7], attention.keep[8]
        self.attn = i16(proj_q.N)
        self.h2, self.act, self.out = i16(hidden), i16(ffn), i16(hidden)
        self.attn_ws = torch.empty(max(attention.workspace_bytes(), 256), dtype=torch.uint8, device=dev)
        all_projs = [proj_q, proj_k, proj_v, proj_o, proj_gate_up, proj_down]
        n_ws = max(B.workspace_bytes(g, M) for g in ([proj_q, proj_k, proj_v], [proj_o], [proj_gate_up], [proj_down]))
        self.ws = torch.zeros(max(n_ws, 256), dtype=torch.uint8, device=dev)
        norm1 = dict(row_scale=self.s1) if h_sq is None else dict(sq_in=h_sq, sq_parts=parts, sq_eps=eps)
        rope = lambda: B.Epilogue(pair_op=B.PAIR_ROPE, rope_cos=rope_cos, rope_sin=rope_sin, **norm1)
        self.qkv = B.LayerPlanFused([proj_q, proj_k, proj_v], [rope(), rope(), B.Epilogue(**norm1)],
                                    [h, h, h], [self.q, self.k_new, self.v_new], row_adapter, M, B.Y_BF16, self.ws)
        self.o = B.LayerPlanFused([proj_o], [B.Epilogue(residual=h, sq_out=self.sq2)], [self.attn], [self.h2],
                                  row_adapter, M, B.Y_BF16, self.ws)
        self.gate_up = B.LayerPlanFused([proj_gate_up],
                                        [B.Epilogue(pair_op=B.PAIR_SWIGLU, sq_in=self.sq2, sq_parts=parts, sq_eps=eps)],
                                        [self.h2], [self.act], row_adapter, M, B.Y_BF16, self.ws)
        self.down = B.LayerPlanFused([proj_down], [B.Epilogue(residual=self.h2, sq_out=self.out_sq)], [self.act],
                                     [self.out], row_adapter, M, B.Y_BF16, self.ws)
        self.keep = (all_projs, rope_cos, rope_sin, row_adapter)
        self.hidden = hidden

    def run(self, stream: Optional[int] = None) -> None:
        if self.h_sq is None:
            B.rms_scale(self.h, self.M, self.hidden, self.eps, self.s1, stream)
        self.qkv.run(stream)
        self.attention.run(self.q, self.attn, B.Y_BF16, self.attn_ws, stream)
        self.o.run(stream)
        self.gate_up.run(stream)
        self.down.run(stream)
