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
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile oracle.c -> liboracle.so (plain gcc, OpenMP over output columns)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
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
