"""Host numpy tensors -> device buffers for the library (plumbing used by tests and bench).

Uploads the canonical tensors of a workloads.Problem, runs the one-time prepack and returns
a binding.Proj.  16-bit float patterns travel as torch.int16, packed codes as torch.uint8.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding


def to_device(a: np.ndarray, device="cuda:0") -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).to(device)


def upload_problem(problem, device="cuda:0", with_lora: bool = True) -> binding.Proj:
    """problem: workloads.Problem (or anything with shape/wq/scales/lora_a/lora_b)."""
    s = problem.shape
    wq = to_device(problem.wq, device)
    scales = to_device(problem.scales, device)
    blob = torch.empty(binding.blob_bytes(s.K, s.N, s.group), dtype=torch.uint8, device=device)
    binding.prepack(s.K, s.N, s.group, wq, scales, blob)
    torch.cuda.synchronize()
    del wq, scales
    if with_lora and s.n_adapters > 0:
        return binding.Proj(s.K, s.N, s.group, blob, to_device(problem.lora_a, device),
                            to_device(problem.lora_b, device), s.alpha)
    return binding.Proj(s.K, s.N, s.group, blob, None, None, s.alpha)


def upload_problem_lora_int16(problem, device="cuda:0") -> binding.Proj:
    """problem: workloads.ProblemLoraInt16 (int16 LoRA stacks aq, bq with scales s_a, s_b).  The
    library expands them into a bf16 pair of four times the rank and folds the scales into alpha."""
    s = problem.shape
    wq = to_device(problem.wq, device)
    scales = to_device(problem.scales, device)
    blob = torch.empty(binding.blob_bytes(s.K, s.N, s.group), dtype=torch.uint8, device=device)
    binding.prepack(s.K, s.N, s.group, wq, scales, blob)
    aq, bq = to_device(problem.aq, device), to_device(problem.bq, device)
    lora_a = torch.empty((s.n_adapters, 4 * s.rank, s.K), dtype=torch.int16, device=device)
    lora_b = torch.empty((s.n_adapters, s.N, 4 * s.rank), dtype=torch.int16, device=device)
    alpha = binding.lora_int16_expand(aq, bq, s.n_adapters, s.rank, s.K, s.N, s.alpha, float(problem.s_a),
                                      float(problem.s_b), lora_a, lora_b)
    torch.cuda.synchronize()
    return binding.Proj(s.K, s.N, s.group, blob, lora_a, lora_b, alpha)


def alloc_y(M: int, N: int, y_dtype: int, device="cuda:0") -> torch.Tensor:
    return torch.empty((M, N), dtype=torch.float32 if y_dtype == binding.Y_FP32 else torch.int16,
                       device=device)


def y_to_numpy(y: torch.Tensor) -> np.ndarray:
    """Device output -> float64 numpy (bf16 patterns widened exactly)."""
    if y.dtype == torch.float32:
        return y.cpu().numpy().astype(np.float64)
    bits = y.cpu().numpy().view(np.uint16).astype(np.uint32) << np.uint32(16)
    return bits.view(np.float32).astype(np.float64)


def alloc_workspace(projs, M: int, device="cuda:0") -> torch.Tensor:
    n = max(binding.workspace_bytes(projs, M), 256)
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    binding.workspace_init(ws)              # completion counters start at zero
    return ws
