"""ctypes front end of the plain-C fp64 oracle (lords_oracle.c).  TEST INFRASTRUCTURE ONLY.

`build()` compiles the C file with gcc (+OpenMP) into oracle/liblords_oracle.so;
the wrappers marshal numpy arrays and call it.  No arithmetic lives here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lords_oracle.c")
_LIB = os.path.join(_HERE, "liblords_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, cl, ci = ctypes.c_void_p, ctypes.c_long, ctypes.c_int
        lib.lords_oracle_threads.restype = ci
        lib.lords_oracle_unpack.argtypes = [vp, vp, cl, cl, ci]
        lib.lords_oracle_dequant.argtypes = [vp, vp, vp, vp, vp, cl, cl, cl, ci]
        lib.lords_oracle_matmul.argtypes = [vp, vp, vp, vp, vp, vp, cl, cl, cl, cl, ci]
        lib.lords_oracle_matmul_rows.argtypes = [vp, vp, vp, vp, vp, vp, cl, cl, cl, cl, ci, vp, cl]
        lib.lords_oracle_pack.argtypes = [vp, vp, cl, cl, ci]
        lib.lords_oracle_quantize_f32.argtypes = [vp, vp, vp, vp, vp, cl, cl, cl, ci]
        lib.lords_oracle_block_init_f32.argtypes = [vp, vp, vp, vp, cl, cl, cl, ci]
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def threads() -> int:
    return int(_load().lords_oracle_threads())


def unpack_codes(codes, K: int, bits: int) -> np.ndarray:
    codes = _c(codes, np.uint8)
    N = codes.shape[0]
    q = np.empty((N, K), dtype=np.uint8)
    if _load().lords_oracle_unpack(_p(codes), _p(q), N, K, bits) != 0:
        raise ValueError("lords_oracle_unpack: bad argument")
    return q


def dequant(codes, codebook, B, A, bits: int) -> np.ndarray:
    codes, codebook, B, A = _c(codes, np.uint8), _c(codebook, np.float32), _c(B, np.float32), _c(A, np.float32)
    N, r = B.shape
    K = A.shape[1]
    assert A.shape[0] == r and codes.shape == (N, K * bits // 8) and codebook.shape == (1 << bits,)
    W = np.empty((N, K), dtype=np.float64)
    if _load().lords_oracle_dequant(_p(codes), _p(codebook), _p(B), _p(A), _p(W), N, K, r, bits) != 0:
        raise ValueError("lords_oracle_dequant: bad argument")
    return W


def matmul(X, codes, codebook, B, A, bits: int, rows=None) -> np.ndarray:
    """Y = X W_hat^T [M, N]; with `rows`, only those out-features: [M, len(rows)]."""
    X = _c(X, np.float32)
    codes, codebook, B, A = _c(codes, np.uint8), _c(codebook, np.float32), _c(B, np.float32), _c(A, np.float32)
    N, r = B.shape
    M, K = X.shape
    assert A.shape == (r, K) and codes.shape == (N, K * bits // 8) and codebook.shape == (1 << bits,)
    if rows is None:
        Y = np.empty((M, N), dtype=np.float64)
        rc = _load().lords_oracle_matmul(_p(X), _p(codes), _p(codebook), _p(B), _p(A), _p(Y), M, N, K, r, bits)
    else:
        rows = _c(rows, np.int64)
        Y = np.empty((M, rows.size), dtype=np.float64)
        rc = _load().lords_oracle_matmul_rows(_p(X), _p(codes), _p(codebook), _p(B), _p(A), _p(Y),
                                              M, N, K, r, bits, _p(rows), rows.size)
    if rc != 0:
        raise ValueError("lords_oracle_matmul: bad argument")
    return Y


def pack_codes(q, bits: int) -> np.ndarray:
    q = _c(q, np.uint8)
    N, K = q.shape
    codes = np.empty((N, K * bits // 8), dtype=np.uint8)
    if _load().lords_oracle_pack(_p(q), _p(codes), N, K, bits) != 0:
        raise ValueError("lords_oracle_pack: bad argument")
    return codes


def quantize_f32(W, codebook, B, A, bits: int) -> np.ndarray:
    """Level indices chosen in fp32, operation by operation as stated in lords_oracle.c."""
    W, codebook, B, A = _c(W, np.float32), _c(codebook, np.float32), _c(B, np.float32), _c(A, np.float32)
    N, K = W.shape
    r = B.shape[1]
    q = np.empty((N, K), dtype=np.uint8)
    if _load().lords_oracle_quantize_f32(_p(W), _p(codebook), _p(B), _p(A), _p(q), N, K, r, bits) != 0:
        raise ValueError("lords_oracle_quantize_f32: bad argument")
    return q


def block_init_f32(W, codebook, r: int, bits: int):
    W, codebook = _c(W, np.float32), _c(codebook, np.float32)
    N, K = W.shape
    B = np.empty((N, r), dtype=np.float32)
    A = np.empty((r, K), dtype=np.float32)
    if _load().lords_oracle_block_init_f32(_p(W), _p(codebook), _p(B), _p(A), N, K, r, bits) != 0:
        raise ValueError("lords_oracle_block_init_f32: bad argument")
    return B, A
