"""ctypes binding of include/mlora_w4.h.  Tensors are torch CUDA(HIP) tensors used as plain
device buffers; work is enqueued on torch's current stream."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmlora_w4.so")
_lib = None

Y_BF16, Y_FP32 = 0, 1

exported_symbols = (
    "mlora_strerror", "mlora_w4_blob_bytes", "mlora_w4_prepack", "mlora_w4_unpack",
    "mlora_group_rows", "mlora_w4_workspace_bytes", "mlora_w4_linear", "mlora_w4_layer_step",
    "mlora_w4_workspace_init", "mlora_w4_workspace_status", "mlora_w4_debug_spin_limit",
    "mlora_w4_layer_step_static", "mlora_w4_layer_step_plan",
    "mlora_tree_attention_workspace_bytes", "mlora_tree_attention",
    "mlora_w4a8_workspace_bytes", "mlora_w4a8_layer_step",
    "mlora_w4_layer_step_fused", "mlora_rms_scale", "mlora_lora_int16_expand",
    "mlora_ds2d_rows", "mlora_ds2d_layout", "mlora_ds2d_workspace_bytes", "mlora_ds2d_step",
)


class MloraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class _ProjStruct(C.Structure):
    _fields_ = [("K", C.c_int32), ("N", C.c_int32), ("group", C.c_int32),
                ("w_blob", C.c_void_p), ("n_adapters", C.c_int32), ("rank", C.c_int32),
                ("lora_a", C.c_void_p), ("lora_b", C.c_void_p), ("alpha", C.c_float)]


class _Ds2dStruct(C.Structure):
    _fields_ = [("n_streams", C.c_int32), ("n_forecast", C.c_int32), ("depth", C.c_int32),
                ("branch", C.c_int32 * 8), ("next_depth", C.c_int32), ("next_branch", C.c_int32 * 8),
                ("vocab", C.c_int32), ("logits_dtype", C.c_int32)]


class _EpilogueStruct(C.Structure):
    _fields_ = [("row_scale", C.c_void_p), ("pair_op", C.c_int32), ("rope_cos", C.c_void_p),
                ("rope_sin", C.c_void_p), ("residual", C.c_void_p), ("sq_in", C.c_void_p),
                ("sq_parts", C.c_int32), ("sq_eps", C.c_float), ("sq_out", C.c_void_p)]


class _TreeAttnStruct(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("n_streams", C.c_int32), ("rows_per_stream", C.c_int32), ("scale", C.c_float),
                ("k_prefill", C.c_void_p), ("v_prefill", C.c_void_p), ("len_prefill", C.c_int32),
                ("k_fprefix", C.c_void_p), ("v_fprefix", C.c_void_p), ("len_fprefix", C.c_int32),
                ("k_stream", C.c_void_p), ("v_stream", C.c_void_p), ("cap_stream", C.c_int32),
                ("len_stream", C.c_void_p),
                ("k_new", C.c_void_p), ("v_new", C.c_void_p),
                ("parent", C.c_void_p), ("is_forecast", C.c_void_p)]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libmlora_w4.so; raises if it is missing (there is no other implementation)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} not built: run __graft_entry__.build() "
                              "(hipcc --offload-arch=gfx950)")
        lib = C.CDLL(_LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        pp = C.POINTER(_ProjStruct)
        lib.mlora_strerror.restype = C.c_char_p
        lib.mlora_strerror.argtypes = [C.c_int]
        lib.mlora_w4_blob_bytes.restype = sz
        lib.mlora_w4_blob_bytes.argtypes = [i32, i32, i32]
        lib.mlora_w4_prepack.restype = C.c_int
        lib.mlora_w4_prepack.argtypes = [i32, i32, i32, vp, vp, vp, vp]
        lib.mlora_w4_unpack.restype = C.c_int
        lib.mlora_w4_unpack.argtypes = [pp, vp, vp, vp]
        lib.mlora_group_rows.restype = C.c_int
        lib.mlora_group_rows.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp]
        lib.mlora_w4_workspace_bytes.restype = sz
        lib.mlora_w4_workspace_bytes.argtypes = [pp, i32, i32]
        lib.mlora_w4_linear.restype = C.c_int
        lib.mlora_w4_linear.argtypes = [pp, vp, vp, i32, vp, i32, vp, sz, vp]
        lib.mlora_w4_layer_step.restype = C.c_int
        lib.mlora_w4_layer_step.argtypes = [pp, i32, C.POINTER(vp), C.POINTER(vp), vp, i32, i32,
                                            vp, sz, vp]
        lib.mlora_w4_layer_step_static.restype = C.c_int
        lib.mlora_w4_layer_step_static.argtypes = [pp, i32, C.POINTER(vp), C.POINTER(vp), vp, i32, i32, vp]
        lib.mlora_w4_workspace_init.restype = C.c_int
        lib.mlora_w4_workspace_init.argtypes = [vp, sz, vp]
        tp = C.POINTER(_TreeAttnStruct)
        lib.mlora_tree_attention_workspace_bytes.restype = sz
        lib.mlora_tree_attention_workspace_bytes.argtypes = [tp]
        lib.mlora_tree_attention.restype = C.c_int
        lib.mlora_tree_attention.argtypes = [tp, vp, vp, i32, vp, sz, vp]
        lib.mlora_w4a8_workspace_bytes.restype = sz
        lib.mlora_w4a8_workspace_bytes.argtypes = [pp, i32, i32]
        lib.mlora_w4a8_layer_step.restype = C.c_int
        lib.mlora_w4a8_layer_step.argtypes = [pp, i32, C.POINTER(vp), C.POINTER(C.c_float), C.POINTER(vp), vp,
                                              i32, i32, vp, sz, vp]
        lib.mlora_w4_layer_step_fused.restype = C.c_int
        lib.mlora_w4_layer_step_fused.argtypes = [pp, C.POINTER(_EpilogueStruct), i32, C.POINTER(vp), C.POINTER(vp),
                                                  vp, i32, i32, vp, sz, vp]
        lib.mlora_rms_scale.restype = C.c_int
        lib.mlora_rms_scale.argtypes = [vp, i32, i32, C.c_float, vp, vp]
        lib.mlora_lora_int16_expand.restype = C.c_int
        lib.mlora_lora_int16_expand.argtypes = [vp, vp, i32, i32, i32, i32, C.c_float, C.c_float, C.c_float,
                                                vp, vp, C.POINTER(C.c_float), vp]
        dp = C.POINTER(_Ds2dStruct)
        ip = C.POINTER(i32)
        lib.mlora_ds2d_rows.restype = C.c_int
        lib.mlora_ds2d_rows.argtypes = [ip, i32, i32, ip, ip]
        lib.mlora_ds2d_layout.restype = C.c_int
        lib.mlora_ds2d_layout.argtypes = [ip, i32, i32, ip, C.POINTER(C.c_uint8), ip]
        lib.mlora_ds2d_workspace_bytes.restype = sz
        lib.mlora_ds2d_workspace_bytes.argtypes = [dp]
        lib.mlora_ds2d_step.restype = C.c_int
        lib.mlora_ds2d_step.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.mlora_w4_workspace_status.restype = C.c_int
        lib.mlora_w4_workspace_status.argtypes = [vp, C.POINTER(i32), vp]
        lib.mlora_w4_debug_spin_limit.restype = i32
        lib.mlora_w4_debug_spin_limit.argtypes = [i32]
        _lib = lib
    return _lib


def strerror(status: int) -> str:
    return load_library().mlora_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise MloraError(status, where)


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream() -> int:
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


class Proj:
    """One projection descriptor; keeps the tensors it points to alive."""

    def __init__(self, K: int, N: int, group: int, w_blob, lora_a=None, lora_b=None,
                 alpha: float = 1.0, n_adapters: Optional[int] = None, rank: Optional[int] = None):
        self.K, self.N, self.group = int(K), int(N), int(group)
        self.w_blob, self.lora_a, self.lora_b = w_blob, lora_a, lora_b
        self.alpha = float(alpha)
        if lora_a is not None:
            self.n_adapters = int(lora_a.shape[0]) if n_adapters is None else int(n_adapters)
            self.rank = int(lora_a.shape[1]) if rank is None else int(rank)
        else:
            self.n_adapters = 0 if n_adapters is None else int(n_adapters)
            self.rank = 0 if rank is None else int(rank)

    def struct(self) -> _ProjStruct:
        return _ProjStruct(self.K, self.N, self.group, _ptr(self.w_blob), self.n_adapters,
                           self.rank, _ptr(self.lora_a), _ptr(self.lora_b), self.alpha)


def _proj_array(projs: Sequence[Proj]):
    arr = (_ProjStruct * len(projs))()
    for i, p in enumerate(projs):
        arr[i] = p.struct()
    return arr


def blob_bytes(K: int, N: int, group: int) -> int:
    return int(load_library().mlora_w4_blob_bytes(K, N, group))


def prepack(K: int, N: int, group: int, wq, scales_f16, w_blob) -> None:
    _check(load_library().mlora_w4_prepack(K, N, group, _ptr(wq), _ptr(scales_f16), _ptr(w_blob),
                                           _stream()), "mlora_w4_prepack")


def unpack(proj: Proj, codes=None, w_f32=None) -> None:
    st = proj.struct()
    _check(load_library().mlora_w4_unpack(C.byref(st), _ptr(codes), _ptr(w_f32), _stream()),
           "mlora_w4_unpack")


def group_rows(row_adapter, M: int, n_adapters: int, perm, seg_adapter, seg_start, n_seg) -> None:
    _check(load_library().mlora_group_rows(_ptr(row_adapter), M, n_adapters, _ptr(perm),
                                           _ptr(seg_adapter), _ptr(seg_start), _ptr(n_seg),
                                           _stream()), "mlora_group_rows")


def workspace_init(workspace) -> None:
    n = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().mlora_w4_workspace_init(_ptr(workspace), n, _stream()),
           "mlora_w4_workspace_init")


def workspace_status(workspace) -> int:
    """Status word of a workspace (0 = no block gave up waiting); waits for the current stream."""
    word = C.c_int32(-1)
    _check(load_library().mlora_w4_workspace_status(_ptr(workspace), C.byref(word), _stream()),
           "mlora_w4_workspace_status")
    return int(word.value)


def debug_spin_limit(limit: int) -> int:
    return int(load_library().mlora_w4_debug_spin_limit(int(limit)))


def workspace_bytes(projs: Sequence[Proj], M: int) -> int:
    arr = _proj_array(projs)
    return int(load_library().mlora_w4_workspace_bytes(arr, len(projs), M))


def layer_step_plan(projs: Sequence[Proj], M: int) -> dict:
    """How the library would run a call over these projections (see mlora_w4_layer_step_plan)."""
    arr = _proj_array(projs)
    info = (C.c_int32 * 5)()
    _check(load_library().mlora_w4_layer_step_plan(arr, len(projs), M, info), "mlora_w4_layer_step_plan")
    return {"launches": info[0], "wide": bool(info[1]), "rows_per_chunk": info[2],
            "grid_x": info[3], "grid_z": info[4]}


def linear(proj: Proj, x, row_adapter, M: int, y, y_dtype: int = Y_BF16, workspace=None) -> None:
    st = proj.struct()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().mlora_w4_linear(C.byref(st), _ptr(x), _ptr(row_adapter), M, _ptr(y),
                                          y_dtype, _ptr(workspace), ws_bytes, _stream()),
           "mlora_w4_linear")


class LayerPlan:
    """Marshalled arguments of a layer_step call, reusable across calls (no per-call Python
    allocation in timing loops)."""

    def __init__(self, projs: Sequence[Proj], xs: Sequence, ys: Sequence, row_adapter, M: int,
                 y_dtype: int, workspace):
        assert len(projs) == len(xs) == len(ys)
        self.keep = (list(projs), list(xs), list(ys), row_adapter, workspace)
        self.n = len(projs)
        self.arr = _proj_array(projs)
        self.xs = (C.c_void_p * self.n)(*[_ptr(x) for x in xs])
        self.ys = (C.c_void_p * self.n)(*[_ptr(y) for y in ys])
        self.rows = _ptr(row_adapter)
        self.M, self.y_dtype = int(M), int(y_dtype)
        self.ws = _ptr(workspace)
        self.ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        self.fn = load_library().mlora_w4_layer_step

    def run(self, stream: Optional[int] = None) -> None:
        st = self.fn(self.arr, self.n, self.xs, self.ys, self.rows, self.M, self.y_dtype,
                     self.ws, self.ws_bytes, _stream() if stream is None else stream)
        if st != 0:
            raise MloraError(st, "mlora_w4_layer_step")


PAIR_NONE, PAIR_ROPE, PAIR_SWIGLU = 0, 1, 2


class Epilogue:
    """What a fused call does to one projection's outputs (mlora_w4_epilogue); keeps its tensors."""

    def __init__(self, row_scale=None, pair_op: int = PAIR_NONE, rope_cos=None, rope_sin=None, residual=None,
                 sq_in=None, sq_parts: int = 0, sq_eps: float = 0.0, sq_out=None):
        self.keep = (row_scale, rope_cos, rope_sin, residual, sq_in, sq_out)
        self.struct = _EpilogueStruct(_ptr(row_scale), pair_op, _ptr(rope_cos), _ptr(rope_sin), _ptr(residual),
                                      _ptr(sq_in), int(sq_parts), float(sq_eps), _ptr(sq_out))


class LayerPlanFused:
    """Marshalled arguments of mlora_w4_layer_step_fused."""

    def __init__(self, projs: Sequence[Proj], epis: Sequence[Epilogue], xs: Sequence, ys: Sequence, row_adapter,
                 M: int, y_dtype: int, workspace):
        assert len(projs) == len(xs) == len(ys) == len(epis)
        self.keep = (list(projs), list(epis), list(xs), list(ys), row_adapter, workspace)
        self.n = len(projs)
        self.arr = _proj_array(projs)
        self.epis = (_EpilogueStruct * self.n)(*[e.struct for e in epis])
        self.xs = (C.c_void_p * self.n)(*[_ptr(x) for x in xs])
        self.ys = (C.c_void_p * self.n)(*[_ptr(y) for y in ys])
        self.rows = _ptr(row_adapter)
        self.M, self.y_dtype = int(M), int(y_dtype)
        self.ws = _ptr(workspace)
        self.ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        self.fn = load_library().mlora_w4_layer_step_fused

    def run(self, stream: Optional[int] = None) -> None:
        st = self.fn(self.arr, self.epis, self.n, self.xs, self.ys, self.rows, self.M, self.y_dtype,
                     self.ws, self.ws_bytes, _stream() if stream is None else stream)
        if st != 0:
            raise MloraError(st, "mlora_w4_layer_step_fused")


def rms_scale(x, M: int, K: int, eps: float, scale, stream: Optional[int] = None) -> None:
    _check(load_library().mlora_rms_scale(_ptr(x), M, K, float(eps), _ptr(scale),
                                          _stream() if stream is None else stream), "mlora_rms_scale")


def lora_int16_expand(a_q, b_q, n_adapters: int, rank: int, K: int, N: int, alpha: float, s_a: float, s_b: float,
                      lora_a, lora_b, stream: Optional[int] = None) -> float:
    """int16 LoRA stacks -> the bf16 tensors of a pair of four times the rank (written to lora_a,
    lora_b); returns the alpha to use with them."""
    alpha_out = C.c_float(0.0)
    _check(load_library().mlora_lora_int16_expand(_ptr(a_q), _ptr(b_q), n_adapters, rank, K, N, float(alpha),
                                                  float(s_a), float(s_b), _ptr(lora_a), _ptr(lora_b),
                                                  C.byref(alpha_out), _stream() if stream is None else stream),
           "mlora_lora_int16_expand")
    return float(alpha_out.value)


def a8_workspace_bytes(projs: Sequence[Proj], M: int) -> int:
    arr = _proj_array(projs)
    return int(load_library().mlora_w4a8_workspace_bytes(arr, len(projs), M))


class LayerPlanA8:
    """Marshalled arguments of mlora_w4a8_layer_step (int8 activations, one scale per tensor)."""

    def __init__(self, projs: Sequence[Proj], xs: Sequence, x_scales: Sequence[float], ys: Sequence,
                 row_adapter, M: int, y_dtype: int, workspace):
        assert len(projs) == len(xs) == len(ys) == len(x_scales)
        self.keep = (list(projs), list(xs), list(ys), row_adapter, workspace)
        self.n = len(projs)
        self.arr = _proj_array(projs)
        self.xs = (C.c_void_p * self.n)(*[_ptr(x) for x in xs])
        self.ys = (C.c_void_p * self.n)(*[_ptr(y) for y in ys])
        self.scales = (C.c_float * self.n)(*[float(v) for v in x_scales])
        self.rows = _ptr(row_adapter)
        self.M, self.y_dtype = int(M), int(y_dtype)
        self.ws = _ptr(workspace)
        self.ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        self.fn = load_library().mlora_w4a8_layer_step

    def run(self, stream: Optional[int] = None) -> None:
        st = self.fn(self.arr, self.n, self.xs, self.scales, self.ys, self.rows, self.M, self.y_dtype,
                     self.ws, self.ws_bytes, _stream() if stream is None else stream)
        if st != 0:
            raise MloraError(st, "mlora_w4a8_layer_step")


def layer_step_static(projs: Sequence[Proj], xs: Sequence, ys: Sequence, row_adapter, M: int,
                      y_dtype: int = Y_BF16) -> None:
    """mlora_w4_layer_step_static: the library's built-in scratch instead of a workspace."""
    n = len(projs)
    assert n == len(xs) == len(ys)
    arr = _proj_array(projs)
    cxs = (C.c_void_p * n)(*[_ptr(x) for x in xs])
    cys = (C.c_void_p * n)(*[_ptr(y) for y in ys])
    _check(load_library().mlora_w4_layer_step_static(arr, n, cxs, cys, _ptr(row_adapter), int(M),
                                                     int(y_dtype), _stream()),
           "mlora_w4_layer_step_static")


def layer_step(projs: Sequence[Proj], xs: Sequence, ys: Sequence, row_adapter, M: int,
               y_dtype: int = Y_BF16, workspace=None) -> None:
    LayerPlan(projs, xs, ys, row_adapter, M, y_dtype, workspace).run()


class TreeAttention:
    """Descriptor of a masked tree attention call (include/mlora_tree_attention.h); keeps the
    tensors it points to alive.  Tensors are torch device tensors in the layouts of the header."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, n_streams: int, rows_per_stream: int,
                 scale: float, k_prefill, v_prefill, k_fprefix, v_fprefix, k_stream, v_stream, len_stream,
                 k_new, v_new, parent, is_forecast, len_prefill: int, len_fprefix: int, cap_stream: int):
        self.keep = (k_prefill, v_prefill, k_fprefix, v_fprefix, k_stream, v_stream, len_stream, k_new, v_new,
                     parent, is_forecast)
        self.shape = (n_streams * rows_per_stream, n_q_heads, head_dim)
        self.struct = _TreeAttnStruct(n_q_heads, n_kv_heads, head_dim, n_streams, rows_per_stream, scale,
                                      _ptr(k_prefill), _ptr(v_prefill), len_prefill,
                                      _ptr(k_fprefix), _ptr(v_fprefix), len_fprefix,
                                      _ptr(k_stream), _ptr(v_stream), cap_stream, _ptr(len_stream),
                                      _ptr(k_new), _ptr(v_new), _ptr(parent), _ptr(is_forecast))

    def workspace_bytes(self) -> int:
        return int(load_library().mlora_tree_attention_workspace_bytes(C.byref(self.struct)))

    def run(self, q, out, out_dtype: int, workspace, stream: Optional[int] = None) -> None:
        n = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(load_library().mlora_tree_attention(C.byref(self.struct), _ptr(q), _ptr(out), out_dtype,
                                                   _ptr(workspace), n, _stream() if stream is None else stream),
               "mlora_tree_attention")


def ds2d_rows(branch: Sequence[int], n_forecast: int):
    """(tokens, rows) of one stream for a branch configuration (mlora_ds2d_rows)."""
    arr = (C.c_int32 * max(1, len(branch)))(*[int(b) for b in branch])
    t, r = C.c_int32(0), C.c_int32(0)
    _check(load_library().mlora_ds2d_rows(arr, len(branch), n_forecast, C.byref(t), C.byref(r)), "mlora_ds2d_rows")
    return int(t.value), int(r.value)


def ds2d_layout(branch: Sequence[int], n_forecast: int):
    """(parent, is_forecast, level) lists of one stream (mlora_ds2d_layout)."""
    _, rows = ds2d_rows(branch, n_forecast)
    arr = (C.c_int32 * max(1, len(branch)))(*[int(b) for b in branch])
    parent, level = (C.c_int32 * rows)(), (C.c_int32 * rows)()
    is_forecast = (C.c_uint8 * rows)()
    _check(load_library().mlora_ds2d_layout(arr, len(branch), n_forecast, parent, is_forecast, level),
           "mlora_ds2d_layout")
    return list(parent), list(is_forecast), list(level)


class Ds2dStep:
    """Descriptor of mlora_ds2d_step (include/mlora_ds2d.h)."""

    def __init__(self, n_streams: int, n_forecast: int, branch: Sequence[int], next_branch: Sequence[int],
                 vocab: int, logits_dtype: int):
        st = _Ds2dStruct()
        st.n_streams, st.n_forecast, st.depth, st.next_depth = n_streams, n_forecast, len(branch), len(next_branch)
        for i, b in enumerate(branch):
            st.branch[i] = int(b)
        for i, b in enumerate(next_branch):
            st.next_branch[i] = int(b)
        st.vocab, st.logits_dtype = vocab, logits_dtype
        self.struct = st

    def workspace_bytes(self) -> int:
        return int(load_library().mlora_ds2d_workspace_bytes(C.byref(self.struct)))

    def run(self, logits, tokens, n_accepted, accepted_rows, emitted, next_tokens, workspace,
            stream: Optional[int] = None) -> None:
        n = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(load_library().mlora_ds2d_step(C.byref(self.struct), _ptr(logits), _ptr(tokens), _ptr(n_accepted),
                                              _ptr(accepted_rows), _ptr(emitted), _ptr(next_tokens),
                                              _ptr(workspace), n, _stream() if stream is None else stream),
               "mlora_ds2d_step")
