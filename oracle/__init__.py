"""ctypes front end of the CPU oracle (oracle.c).  TEST INFRASTRUCTURE ONLY.

Imported by the tests, the smoke check and the benchmark's cpu_baseline leg;
never by the HIP library or its Python binding.  All arithmetic lives in
oracle.c; this file only compiles it with gcc, marshals numpy arrays and
reshapes results.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "oracle.c"), os.path.join(_HERE, "tree_attention.c"),
         os.path.join(_HERE, "act_quant.c")]
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c and tree_attention.c -> liboracle.so (plain gcc, OpenMP over output columns)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-o", _LIB, *_SRCS, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        u8p, u16p, i8p, i32p, f32p, f64p = (C.POINTER(t) for t in
                                            (C.c_uint8, C.c_uint16, C.c_int8, C.c_int32,
                                             C.c_float, C.c_double))
        i32 = C.c_int32
        lib.orc_bf16_to_double.restype = C.c_double
        lib.orc_bf16_to_double.argtypes = [C.c_uint16]
        lib.orc_f16_to_double.restype = C.c_double
        lib.orc_f16_to_double.argtypes = [C.c_uint16]
        lib.orc_f32_to_f16.restype = C.c_uint16
        lib.orc_f32_to_f16.argtypes = [C.c_float]
        lib.orc_unpack_codes.argtypes = [u8p, i32, i32, i8p]
        lib.orc_pack_codes.argtypes = [i8p, i32, i32, u8p]
        lib.orc_dequant.argtypes = [u8p, u16p, i32, i32, i32, f64p]
        lib.orc_quantise.argtypes = [f32p, i32, i32, i32, u8p, u16p]
        lib.orc_group_rows.restype = i32
        lib.orc_group_rows.argtypes = [i32p, i32, i32, i32p, i32p, i32p, i32p]
        lib.orc_set_threads.argtypes = [i32]
        lib.orc_max_threads.restype = i32
        lib.orc_linear.argtypes = [i32, i32, i32, u8p, u16p, i32, i32, u16p, u16p, C.c_double,
                                   u16p, i32p, i32, f64p, f64p]
        lib.orc_linear_a8.argtypes = [i32, i32, i32, u8p, u16p, i32, u16p, u16p, C.c_double,
                                      i8p, C.c_double, i32p, i32, f64p]
        lib.orc_linear_a8.restype = None
        lib.orc_quantise_act.argtypes = [f32p, C.c_size_t, i8p]
        lib.orc_quantise_act.restype = C.c_float
        lib.orc_tree_attention.restype = i32
        lib.orc_tree_attention.argtypes = [i32, i32, i32, i32, i32, C.c_double,
                                           u16p, u16p, i32, u16p, u16p, i32, u16p, u16p, i32, i32p,
                                           u16p, u16p, i32p, u8p, u16p, f64p, f64p]
        for f in (lib.orc_unpack_codes, lib.orc_pack_codes, lib.orc_dequant, lib.orc_quantise,
                  lib.orc_set_threads, lib.orc_linear):
            f.restype = None
        _lib = lib
    return _lib


def _p(a: np.ndarray, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _arr(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.dtype(dtype):
        raise TypeError(f"expected {np.dtype(dtype)}, got {a.dtype}")
    return a


def bf16_to_double(bits: int) -> float:
    return float(_load().orc_bf16_to_double(int(bits)))


def f16_to_double(bits: int) -> float:
    return float(_load().orc_f16_to_double(int(bits)))


def f32_to_f16(value: float) -> int:
    return int(_load().orc_f32_to_f16(float(value)))


def unpack_codes(wq: np.ndarray) -> np.ndarray:
    wq = _arr(wq, np.uint8)
    N, K = wq.shape[0], wq.shape[1] * 2
    codes = np.empty((N, K), np.int8)
    _load().orc_unpack_codes(_p(wq, C.c_uint8), N, K, _p(codes, C.c_int8))
    return codes


def pack_codes(codes: np.ndarray) -> np.ndarray:
    codes = _arr(codes, np.int8)
    N, K = codes.shape
    wq = np.empty((N, K // 2), np.uint8)
    _load().orc_pack_codes(_p(codes, C.c_int8), N, K, _p(wq, C.c_uint8))
    return wq


def dequant(wq: np.ndarray, scales: np.ndarray, group: int) -> np.ndarray:
    wq, scales = _arr(wq, np.uint8), _arr(scales, np.uint16)
    N, K = wq.shape[0], wq.shape[1] * 2
    assert scales.shape == (N, K // group)
    w = np.empty((N, K), np.float64)
    _load().orc_dequant(_p(wq, C.c_uint8), _p(scales, C.c_uint16), N, K, group, _p(w, C.c_double))
    return w


def quantise(w: np.ndarray, group: int):
    w = _arr(w, np.float32)
    N, K = w.shape
    wq = np.zeros((N, K // 2), np.uint8)
    scales = np.empty((N, K // group), np.uint16)
    _load().orc_quantise(_p(w, C.c_float), N, K, group, _p(wq, C.c_uint8), _p(scales, C.c_uint16))
    return wq, scales


def group_rows(row_adapter: np.ndarray, n_adapters: int):
    """-> (perm[M], seg_adapter[U], seg_start[U+1]); raises ValueError on an index out of range."""
    ra = _arr(row_adapter, np.int32)
    M = ra.shape[0]
    perm = np.empty(max(M, 1), np.int32)
    seg_adapter = np.empty(max(n_adapters, 1), np.int32)
    seg_start = np.empty(n_adapters + 1, np.int32)
    n_seg = C.c_int32(0)
    rc = _load().orc_group_rows(_p(ra, C.c_int32), M, n_adapters, _p(perm, C.c_int32),
                                _p(seg_adapter, C.c_int32), _p(seg_start, C.c_int32),
                                C.byref(n_seg))
    if rc != 0:
        raise ValueError("row_adapter index outside [-1, n_adapters)")
    u = n_seg.value
    return perm[:M].copy(), seg_adapter[:u].copy(), seg_start[:u + 1].copy()


def set_threads(n: int) -> None:
    _load().orc_set_threads(int(n))


def max_threads() -> int:
    return int(_load().orc_max_threads())


def linear(wq, scales, group, lora_a, lora_b, alpha, x, row_adapter, return_t: bool = False):
    """y[M][N] in float64 for one projection (and t[M][rank] if asked)."""
    wq, scales = _arr(wq, np.uint8), _arr(scales, np.uint16)
    lora_a, lora_b = _arr(lora_a, np.uint16), _arr(lora_b, np.uint16)
    x = _arr(x, np.uint16)
    N, K = wq.shape[0], wq.shape[1] * 2
    M = x.shape[0]
    n_adapters, rank = lora_a.shape[0], lora_a.shape[1]
    assert x.shape == (M, K) and scales.shape == (N, K // group)
    assert lora_a.shape == (n_adapters, rank, K) and lora_b.shape == (n_adapters, N, rank)
    ra = None if row_adapter is None else _arr(row_adapter, np.int32)
    if ra is not None:
        assert ra.shape == (M,)
        if ra.size and (ra.min() < -1 or ra.max() >= n_adapters):
            raise ValueError("row_adapter index outside [-1, n_adapters)")
    y = np.empty((M, N), np.float64)
    t = np.zeros((M, rank), np.float64)
    _load().orc_linear(K, N, group, _p(wq, C.c_uint8), _p(scales, C.c_uint16), n_adapters, rank,
                       _p(lora_a, C.c_uint16), _p(lora_b, C.c_uint16), float(alpha),
                       _p(x, C.c_uint16), None if ra is None else _p(ra, C.c_int32), M,
                       _p(y, C.c_double), _p(t, C.c_double))
    return (y, t) if return_t else y


def linear_a8(wq, scales, group, lora_a, lora_b, alpha, xq, x_scale, row_adapter):
    """y[M][N] in float64 for one projection on int8 activations xq [M][K] with scale x_scale
    (act_quant.c)."""
    wq, scales = _arr(wq, np.uint8), _arr(scales, np.uint16)
    lora_a, lora_b = _arr(lora_a, np.uint16), _arr(lora_b, np.uint16)
    xq = _arr(xq, np.int8)
    N, K = wq.shape[0], wq.shape[1] * 2
    M = xq.shape[0]
    n_adapters, rank = lora_a.shape[0], lora_a.shape[1]
    assert xq.shape == (M, K) and scales.shape == (N, K // group)
    assert lora_a.shape == (n_adapters, rank, K) and lora_b.shape == (n_adapters, N, rank)
    ra = None if row_adapter is None else _arr(row_adapter, np.int32)
    if ra is not None:
        assert ra.shape == (M,)
        if ra.size and (ra.min() < -1 or ra.max() >= n_adapters):
            raise ValueError("row_adapter index outside [-1, n_adapters)")
    y = np.empty((M, N), np.float64)
    _load().orc_linear_a8(K, N, group, _p(wq, C.c_uint8), _p(scales, C.c_uint16), rank,
                          _p(lora_a, C.c_uint16), _p(lora_b, C.c_uint16), float(alpha),
                          _p(xq, C.c_int8), float(x_scale), None if ra is None else _p(ra, C.c_int32), M,
                          _p(y, C.c_double))
    return y


def quantise_act(x):
    """(xq int8, scale float32) of a float32 tensor: one scale per tensor (act_quant.c)."""
    x = _arr(x, np.float32)
    xq = np.empty(x.shape, np.int8)
    scale = _load().orc_quantise_act(_p(x, C.c_float), x.size, _p(xq, C.c_int8))
    return xq, np.float32(scale)


def tree_attention(q, k_prefill, v_prefill, k_fprefix, v_fprefix, k_stream, v_stream, len_stream,
                   k_new, v_new, parent, is_forecast, n_streams: int, scale: float,
                   return_weights: bool = False):
    """Masked tree attention over a segmented KV cache (tree_attention.c).  bf16 tensors as uint16:
    q [M][Hq][D]; k_prefill, v_prefill [Hkv][Lp][D]; k_fprefix, v_fprefix [Hkv][Lf][D];
    k_stream, v_stream [S][Hkv][cap][D]; len_stream int32 [S]; k_new, v_new [M][Hkv][D];
    parent int32 [M] (index within the stream, -1 = root); is_forecast uint8 [M].
    Returns out float64 [M][Hq][D] (and the weights [M][Hq][Lp + Lf + cap + R] if asked)."""
    q = _arr(q, np.uint16)
    M, Hq, D = q.shape
    S = int(n_streams)
    assert M % S == 0
    R = M // S
    k_prefill, v_prefill = _arr(k_prefill, np.uint16), _arr(v_prefill, np.uint16)
    k_fprefix, v_fprefix = _arr(k_fprefix, np.uint16), _arr(v_fprefix, np.uint16)
    k_stream, v_stream = _arr(k_stream, np.uint16), _arr(v_stream, np.uint16)
    k_new, v_new = _arr(k_new, np.uint16), _arr(v_new, np.uint16)
    Hkv, Lp = k_prefill.shape[0], k_prefill.shape[1]
    Lf, cap = k_fprefix.shape[1], k_stream.shape[2]
    assert Hq % Hkv == 0
    assert k_prefill.shape == v_prefill.shape == (Hkv, Lp, D)
    assert k_fprefix.shape == v_fprefix.shape == (Hkv, Lf, D)
    assert k_stream.shape == v_stream.shape == (S, Hkv, cap, D)
    assert k_new.shape == v_new.shape == (M, Hkv, D)
    len_stream = _arr(len_stream, np.int32)
    parent, is_forecast = _arr(parent, np.int32), _arr(is_forecast, np.uint8)
    assert len_stream.shape == (S,) and parent.shape == (M,) and is_forecast.shape == (M,)
    assert len_stream.min(initial=0) >= 0 and len_stream.max(initial=0) <= cap
    out = np.empty((M, Hq, D), np.float64)
    weights = np.zeros((M, Hq, Lp + Lf + cap + R), np.float64) if return_weights else None
    u16 = C.c_uint16
    rc = _load().orc_tree_attention(Hq, Hkv, D, S, R, float(scale),
                                    _p(k_prefill, u16), _p(v_prefill, u16), Lp,
                                    _p(k_fprefix, u16), _p(v_fprefix, u16), Lf,
                                    _p(k_stream, u16), _p(v_stream, u16), cap, _p(len_stream, C.c_int32),
                                    _p(k_new, u16), _p(v_new, u16), _p(parent, C.c_int32),
                                    _p(is_forecast, C.c_uint8), _p(q, u16), _p(out, C.c_double),
                                    None if weights is None else _p(weights, C.c_double))
    if rc != 0:
        raise ValueError("parent[] must point to an earlier row of the same stream, or be -1")
    return (out, weights) if return_weights else out
