"""ctypes front end of the plain-C oracle.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this module.  It imports nothing from the HIP package and the HIP package
imports nothing from here.  All arithmetic lives in vlut_oracle.c; this file
marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vlut_oracle.c")
_LIB = os.path.join(_HERE, "libvlut_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, IEEE arithmetic, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        i64, p = ctypes.c_int64, ctypes.c_void_p
        _lib.oracle_get_sign.argtypes = [ctypes.c_int] * 3
        _lib.oracle_get_sign.restype = ctypes.c_int
        _lib.oracle_pack_indices.argtypes = [p, i64, i64, ctypes.c_int, p]
        _lib.oracle_unpack_indices.argtypes = [p, i64, i64, ctypes.c_int, p]
        _lib.oracle_quantize.argtypes = [p, i64, i64, i64, p, p]
        _lib.oracle_quantize.restype = None
        _lib.oracle_gemm_acc.argtypes = [p, p, i64, i64, i64, p]
        _lib.oracle_epilogue.argtypes = [p, i64, i64, ctypes.c_float, p, p, i64]
        _lib.oracle_epilogue.restype = None
        _lib.oracle_build_lut.argtypes = [p, i64, i64, ctypes.c_int, p]
        _lib.oracle_build_lut.restype = None
        _lib.oracle_lookup_accumulate.argtypes = [p, p, i64, i64, i64, ctypes.c_int, p]
        _lib.oracle_lookup_accumulate.restype = None
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def get_sign(i: int, j: int, g: int = 4) -> int:
    return _load().oracle_get_sign(i, j, g)


def pack_indices(W: np.ndarray, g: int = 4) -> np.ndarray:
    W = _c(W, np.int8)
    M, K = W.shape
    assert K % g == 0
    idx = np.empty((M, K // g), dtype=np.uint8)
    rc = _load().oracle_pack_indices(_ptr(W), M, K, g, _ptr(idx))
    if rc != 0:
        raise ValueError("weight outside {-1,0,+1}")
    return idx


def unpack_indices(idx: np.ndarray, g: int = 4) -> np.ndarray:
    idx = _c(idx, np.uint8)
    M, G = idx.shape
    W = np.empty((M, G * g), dtype=np.int8)
    rc = _load().oracle_unpack_indices(_ptr(idx), M, G * g, g, _ptr(W))
    if rc != 0:
        raise ValueError("index outside [0, 3^g)")
    return W


def quantize(x: np.ndarray):
    """x fp32 [N][K] (any row stride) -> (q int8 [K][N], s fp32 [N])."""
    assert x.dtype == np.float32 and x.ndim == 2 and x.strides[1] == 4
    N, K = x.shape
    ldx = x.strides[0] // 4
    q = np.empty((K, N), dtype=np.int8)
    s = np.empty(N, dtype=np.float32)
    _load().oracle_quantize(_ptr(x), N, K, ldx, _ptr(q), _ptr(s))
    return q, s


def gemm_acc(W: np.ndarray, q: np.ndarray) -> np.ndarray:
    W = _c(W, np.int8)
    q = _c(q, np.int8)
    M, K = W.shape
    K2, N = q.shape
    assert K == K2
    acc = np.empty((M, N), dtype=np.int32)
    rc = _load().oracle_gemm_acc(_ptr(W), _ptr(q), M, K, N, _ptr(acc))
    if rc == 1:
        raise ValueError("weight outside {-1,0,+1}")
    if rc == 2:
        raise OverflowError("accumulator does not fit INT32")
    return acc


def epilogue(acc: np.ndarray, w_scale, s: np.ndarray) -> np.ndarray:
    """fp64 y [N][M] = acc[m][n] * w_scale * s[n]."""
    acc = _c(acc, np.int32)
    s = _c(s, np.float32)
    M, N = acc.shape
    y = np.empty((N, M), dtype=np.float64)
    _load().oracle_epilogue(_ptr(acc), M, N, ctypes.c_float(float(np.float32(w_scale))), _ptr(s),
                            _ptr(y), M)
    return y


def build_lut(q: np.ndarray, g: int = 4) -> np.ndarray:
    q = _c(q, np.int8)
    K, N = q.shape
    assert K % g == 0
    T = np.empty((K // g, 3 ** g, N), dtype=np.int16)
    _load().oracle_build_lut(_ptr(q), K, N, g, _ptr(T))
    return T


def lookup_accumulate(idx: np.ndarray, T: np.ndarray, g: int = 4) -> np.ndarray:
    idx = _c(idx, np.uint8)
    T = _c(T, np.int16)
    M, G = idx.shape
    N = T.shape[2]
    assert T.shape[0] == G and T.shape[1] == 3 ** g
    acc = np.empty((M, N), dtype=np.int32)
    _load().oracle_lookup_accumulate(_ptr(idx), _ptr(T), M, G * g, N, g, _ptr(acc))
    return acc


def mpgemm(W: np.ndarray, w_scale, x: np.ndarray):
    """Whole path: quantise, integer GEMM, scale.  Returns (q, s, acc, y)."""
    q, s = quantize(np.ascontiguousarray(x, dtype=np.float32))
    acc = gemm_acc(W, q)
    return q, s, acc, epilogue(acc, w_scale, s)


def num_threads() -> int:
    return _load().oracle_num_threads()
