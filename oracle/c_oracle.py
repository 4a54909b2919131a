"""Build and call the plain-C oracle (oracle/lqq_oracle.c).  TEST INFRASTRUCTURE ONLY.

`build()` compiles the C file with gcc (-O3 -fopenmp, no intrinsics, no BLAS) into
oracle/liblqq_oracle.so; the wrappers below marshal numpy arrays.  Nothing here is
shared with, or imported by, the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lqq_oracle.c")
_LIB = os.path.join(_HERE, "liblqq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_int, vp = ctypes.c_int, ctypes.c_void_p
        lib.lqq_oracle_threads.restype = c_int
        lib.lqq_oracle_dequant.restype = c_int
        lib.lqq_oracle_dequant.argtypes = [c_int, c_int, c_int, vp, vp, vp, vp]
        lib.lqq_oracle_matmul_scale.restype = c_int
        lib.lqq_oracle_matmul_scale.argtypes = [c_int, c_int, c_int, vp, vp, vp, vp, vp, vp]
        lib.lqq_oracle_w4a8_gemm.restype = c_int
        lib.lqq_oracle_w4a8_gemm.argtypes = [c_int] * 4 + [vp] * 8
        _lib = lib
    return _lib


def _p(arr):
    return arr.ctypes.data_as(ctypes.c_void_p)


def threads() -> int:
    return int(_load().lqq_oracle_threads())


def dequant(packed, s_u8, a, g):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    s_u8 = np.ascontiguousarray(s_u8, dtype=np.uint8)
    a = np.ascontiguousarray(a, dtype=np.uint8)
    N, K = packed.shape[0], packed.shape[1] * 2
    Wd = np.empty((N, K), dtype=np.int8)
    rc = _load().lqq_oracle_dequant(N, K, g, _p(packed), _p(s_u8), _p(a), _p(Wd))
    if rc != 0:
        raise ArithmeticError(f"lqq_oracle_dequant failed: {rc}")
    return Wd


def matmul_scale(X_i8, s_x, Wd, s_w, want_y=True):
    X_i8 = np.ascontiguousarray(X_i8, dtype=np.int8)
    Wd = np.ascontiguousarray(Wd, dtype=np.int8)
    s_x = np.ascontiguousarray(s_x, dtype=np.float32)
    s_w = np.ascontiguousarray(s_w, dtype=np.float32)
    M, K = X_i8.shape
    N = Wd.shape[0]
    assert Wd.shape[1] == K and s_x.shape == (M,) and s_w.shape == (N,)
    ACC = np.empty((M, N), dtype=np.int32)
    Y = np.empty((M, N), dtype=np.float64) if want_y else None
    rc = _load().lqq_oracle_matmul_scale(M, N, K, _p(X_i8), _p(s_x), _p(Wd), _p(s_w), _p(ACC),
                                         _p(Y) if want_y else None)
    if rc != 0:
        raise ArithmeticError(f"lqq_oracle_matmul_scale failed: {rc}")
    if not want_y:
        return ACC, None
    with np.errstate(over="ignore"):
        return ACC, Y.astype(np.float16)


def w4a8_gemm(X_i8, s_x, packed, s_u8, a, s_w, g):
    """Whole path in C; returns (ACC int32, Y float16 rounded once from double)."""
    X_i8 = np.ascontiguousarray(X_i8, dtype=np.int8)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    s_u8 = np.ascontiguousarray(s_u8, dtype=np.uint8)
    a = np.ascontiguousarray(a, dtype=np.uint8)
    s_x = np.ascontiguousarray(s_x, dtype=np.float32)
    s_w = np.ascontiguousarray(s_w, dtype=np.float32)
    M, K = X_i8.shape
    N = packed.shape[0]
    assert packed.shape[1] * 2 == K
    ACC = np.empty((M, N), dtype=np.int32)
    Y = np.empty((M, N), dtype=np.float64)
    rc = _load().lqq_oracle_w4a8_gemm(M, N, K, g, _p(X_i8), _p(s_x), _p(packed), _p(s_u8), _p(a),
                                      _p(s_w), _p(ACC), _p(Y))
    if rc != 0:
        raise ArithmeticError(f"lqq_oracle_w4a8_gemm failed: {rc}")
    with np.errstate(over="ignore"):
        return ACC, Y.astype(np.float16)


if __name__ == "__main__":
    print(build(force=True))
