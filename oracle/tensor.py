"""TEST INFRASTRUCTURE ONLY: ctypes front end of the fp64 CPU tensor oracle.

The arithmetic lives in ``tensor_oracle.c`` (plain nested loops, one fp64
accumulator per output element).  This module only compiles that file with gcc
when the shared object is missing or older than the source, loads it, and
marshals numpy arrays.  Nothing here imports the product package, and the
product package never imports this.

Operators (App. B.1, B.2, B.3 / Eq. 5):
    matmul(A[M,K], B[K,N])                     -> C[M,N]
    bmm(A[b,M,K], B[b,K,N])                    -> C[b,M,N]
    conv2d(img[B,Cin,H,W], ker[Cout,Cin,Hk,Wk], stride, pad) -> out[B,Cout,Hout,Wout]
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tensor_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_tensor.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile tensor_oracle.c with gcc (+OpenMP); returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-o", tmp, _SRC]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            i64 = ctypes.c_int64
            dp = ctypes.POINTER(ctypes.c_double)
            ip = ctypes.POINTER(ctypes.c_int64)
            lib.oracle_num_threads.restype = ctypes.c_int
            lib.oracle_set_threads.argtypes = [ctypes.c_int]
            lib.oracle_matmul.argtypes = [dp, dp, dp, i64, i64, i64]
            lib.oracle_matmul_rows.argtypes = [dp, dp, dp, ip, i64, i64, i64]
            lib.oracle_matmul_entries.argtypes = [dp, dp, dp, ip, ip, i64, i64, i64]
            lib.oracle_bmm.argtypes = [dp, dp, dp, i64, i64, i64, i64]
            lib.oracle_conv_out_extent.argtypes = [i64, i64, i64, i64]
            lib.oracle_conv_out_extent.restype = i64
            lib.oracle_conv2d.argtypes = [dp, dp, dp] + [i64] * 9
            _lib = lib
    return _lib


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ip(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def matmul(A, B) -> np.ndarray:
    A, B = _f64(A), _f64(B)
    assert A.ndim == 2 and B.ndim == 2 and A.shape[1] == B.shape[0]
    M, K = A.shape
    N = B.shape[1]
    C = np.empty((M, N), dtype=np.float64)
    _load().oracle_matmul(_dp(A), _dp(B), _dp(C), M, N, K)
    return C


def matmul_rows(A, B, rows) -> np.ndarray:
    """Full rows ``rows`` of A.B, each entry by the plain sum."""
    A, B = _f64(A), _f64(B)
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    assert rows.ndim == 1 and (rows >= 0).all() and (rows < A.shape[0]).all()
    K = A.shape[1]
    N = B.shape[1]
    out = np.empty((rows.size, N), dtype=np.float64)
    _load().oracle_matmul_rows(_dp(A), _dp(B), _dp(out), _ip(rows), rows.size, N, K)
    return out


def matmul_entries(A, B, is_, js) -> np.ndarray:
    """Single entries (is_[e], js[e]) of A.B, each by the plain sum."""
    A, B = _f64(A), _f64(B)
    is_ = np.ascontiguousarray(np.asarray(is_, dtype=np.int64))
    js = np.ascontiguousarray(np.asarray(js, dtype=np.int64))
    assert is_.shape == js.shape and is_.ndim == 1
    assert (is_ >= 0).all() and (is_ < A.shape[0]).all()
    assert (js >= 0).all() and (js < B.shape[1]).all()
    out = np.empty(is_.size, dtype=np.float64)
    _load().oracle_matmul_entries(_dp(A), _dp(B), _dp(out), _ip(is_), _ip(js), is_.size,
                                  B.shape[1], A.shape[1])
    return out


def bmm(A, B) -> np.ndarray:
    A, B = _f64(A), _f64(B)
    assert A.ndim == 3 and B.ndim == 3 and A.shape[0] == B.shape[0] and A.shape[2] == B.shape[1]
    b, M, K = A.shape
    N = B.shape[2]
    C = np.empty((b, M, N), dtype=np.float64)
    _load().oracle_bmm(_dp(A), _dp(B), _dp(C), b, M, N, K)
    return C


def conv_out_extent(n_in: int, k: int, stride: int, pad: int) -> int:
    return int(_load().oracle_conv_out_extent(n_in, k, stride, pad))


def conv2d(img, ker, stride: int = 1, pad: int = 0) -> np.ndarray:
    img, ker = _f64(img), _f64(ker)
    assert img.ndim == 4 and ker.ndim == 4 and img.shape[1] == ker.shape[1]
    B, Cin, H, W = img.shape
    Cout, _, Hk, Wk = ker.shape
    Ho = conv_out_extent(H, Hk, stride, pad)
    Wo = conv_out_extent(W, Wk, stride, pad)
    out = np.empty((B, Cout, Ho, Wo), dtype=np.float64)
    _load().oracle_conv2d(_dp(img), _dp(ker), _dp(out), B, Cin, H, W, Cout, Hk, Wk, stride, pad)
    return out
