"""Seeded synthetic inputs shaped like the paper's workloads.

This package only *makes inputs* (shapes, random draws, dtype encodings, the
int4 weight quantiser that turns Gaussian weights into packed codes + scales).
It holds none of the arithmetic of the linear layer itself and imports neither
the CPU oracle nor the HIP library; both consume what it produces.
"""
from .configs import (ProjShape, Workload, WORKLOADS, llama1b_layer_shapes,
                      ds2d_rows, algorithmic_bytes, algorithmic_flops)
from .generate import (Problem, make_problem, make_layer, make_layer_inputs, make_rows,
                       f32_to_bf16_bits, bf16_bits_to_f32, quantise_int4,
                       pack_nibbles, quantise_act_int8, make_x_int8, fuse_gate_up, make_x,
                       quantise_lora_int16, ProblemLoraInt16, make_problem_lora_int16)

from .attention import (AttentionInputs, chain_tree, ds2d_tree, make_attention_inputs, random_tree)

__all__ = [
    "quantise_act_int8", "make_x_int8", "fuse_gate_up", "make_x",
    "quantise_lora_int16", "ProblemLoraInt16", "make_problem_lora_int16",
    "AttentionInputs", "chain_tree", "ds2d_tree", "make_attention_inputs", "random_tree",
    "ProjShape", "Workload", "WORKLOADS", "llama1b_layer_shapes", "ds2d_rows",
    "algorithmic_bytes", "algorithmic_flops", "Problem", "make_problem",
    "make_layer", "make_layer_inputs", "make_rows", "f32_to_bf16_bits", "bf16_bits_to_f32",
    "quantise_int4", "pack_nibbles",
]
