"""mlora_w4 for MI355X: Python binding of the C-ABI library (argument marshalling only).

Every step of the computation runs in the HIP kernels of libmlora_w4.so; nothing here has a
CPU fallback.  Loading fails loudly if the library has not been built
(python -c "import __graft_entry__ as g; g.build()").
"""
from .binding import (lora_int16_expand, Epilogue, LayerPlanFused, rms_scale, PAIR_NONE, PAIR_ROPE, PAIR_SWIGLU, LayerPlanA8, a8_workspace_bytes, Ds2dStep, ds2d_layout, ds2d_rows, LayerPlan, MloraError, Proj, TreeAttention, blob_bytes, group_rows, layer_step, layer_step_plan, layer_step_static,
                      lib_path, linear,
                      load_library, prepack, strerror, unpack, workspace_bytes,
                      Y_BF16, Y_FP32, workspace_init, workspace_status, debug_spin_limit,
                      exported_symbols)

__all__ = ["lora_int16_expand", "Epilogue", "LayerPlanFused", "rms_scale", "PAIR_NONE", "PAIR_ROPE", "PAIR_SWIGLU", "LayerPlanA8", "a8_workspace_bytes", "Ds2dStep", "ds2d_layout", "ds2d_rows", "LayerPlan", "MloraError", "Proj", "TreeAttention", "blob_bytes", "group_rows", "layer_step", "layer_step_plan", "layer_step_static", "lib_path", "linear",
           "load_library", "prepack", "strerror", "unpack", "workspace_bytes", "Y_BF16",
           "Y_FP32", "workspace_init", "workspace_status", "debug_spin_limit", "exported_symbols"]
