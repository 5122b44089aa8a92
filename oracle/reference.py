"""ctypes front end of the C oracle (oracle/gemm_oracle.c).

TEST INFRASTRUCTURE ONLY -- see the package docstring.

The three exported products are the ones an FC layer performs (paper Sec. IV-A,
paragraph introducing the three matrix multiplies; Algorithm 1 lines 3, 11, 13).
Operands are numpy uint16 arrays holding bf16 bit patterns, row-major; results
are numpy float64 arrays (never rounded to bf16).  The storage mode of the two
operands (Sec. IV-C: NN, NT, TN) is passed by name:

    NN: first operand [M,K], second [K,N]
    NT: first operand [M,K], second [N,K]   (second is stored transposed)
    TN: first operand [K,M], second [K,N]   (first is stored transposed)
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_oracle.c")
_SRC_T = os.path.join(_HERE, "transpose_oracle.c")
_LIB = os.path.join(_HERE, "libgemm_oracle.so")

LAYOUTS = {"NN": 0, "NT": 1, "TN": 2}

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no GPU toolchain involved)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_T))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-fopenmp", "-std=c11", "-shared", "-fPIC",
               "-Wall", "-Wextra", _SRC, _SRC_T, "-o", _LIB]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.oracle_gemm_bf16_f64.argtypes = [i64, i64, i64, ctypes.c_int, p, p, p, ctypes.c_int]
        lib.oracle_gemm_bf16_f64.restype = ctypes.c_int
        lib.oracle_gemm_bf16_f64_at.argtypes = [i64, i64, i64, ctypes.c_int, p, p, i64, p, p, p,
                                                ctypes.c_int]
        lib.oracle_gemm_bf16_f64_at.restype = ctypes.c_int
        lib.oracle_transpose_u16.argtypes = [i64, i64, p, p]
        lib.oracle_transpose_u16.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    """Host threads the oracle uses by default: the cores this process may run on."""
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:  # pragma: no cover
        return max(1, os.cpu_count() or 1)


def _operand_shapes(M, N, K, layout):
    if layout == "NN":
        return (M, K), (K, N)
    if layout == "NT":
        return (M, K), (N, K)
    if layout == "TN":
        return (K, M), (K, N)
    raise ValueError(f"unknown layout {layout!r}")


def _check(arr, shape, name):
    if not isinstance(arr, np.ndarray) or arr.dtype != np.uint16:
        raise TypeError(f"{name}: expected a numpy uint16 array of bf16 bit patterns")
    if tuple(arr.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {arr.shape} does not match {shape}")
    return np.ascontiguousarray(arr)


def gemm(M, N, K, layout, A, B, threads=None):
    """C[M,N] (fp64) = sum_k a(i,k) b(k,j), operands stored as `layout` says."""
    sa, sb = _operand_shapes(M, N, K, layout)
    A = _check(A, sa, "A")
    B = _check(B, sb, "B")
    C = np.empty((M, N), dtype=np.float64)
    rc = _load().oracle_gemm_bf16_f64(M, N, K, LAYOUTS[layout], A.ctypes.data, B.ctypes.data,
                                      C.ctypes.data, threads or max_threads())
    if rc != 0:
        raise RuntimeError(f"oracle_gemm_bf16_f64 failed with {rc}")
    return C


def gemm_at(M, N, K, layout, A, B, ii, jj, threads=None):
    """The same product evaluated only at positions (ii[s], jj[s]); returns fp64 [len(ii)]."""
    sa, sb = _operand_shapes(M, N, K, layout)
    A = _check(A, sa, "A")
    B = _check(B, sb, "B")
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    if ii.shape != jj.shape or ii.ndim != 1:
        raise ValueError("ii and jj must be 1-D and of equal length")
    out = np.empty(ii.shape[0], dtype=np.float64)
    rc = _load().oracle_gemm_bf16_f64_at(M, N, K, LAYOUTS[layout], A.ctypes.data, B.ctypes.data,
                                         ii.shape[0], ii.ctypes.data, jj.ctypes.data,
                                         out.ctypes.data, threads or max_threads())
    if rc != 0:
        raise RuntimeError(f"oracle_gemm_bf16_f64_at failed with {rc}")
    return out


def linear_fwd(M, N, K, layout, X, W, threads=None):
    """Forward, Algorithm 1 line 3: O = I x W.  M = tokens, N = out features, K = in features.

    With the buffers the method caches (I as [tokens,in], W as [in,out]) the mode is NN.
    """
    return gemm(M, N, K, layout, X, W, threads)


def linear_bwd_data(M, N, K, layout, dY, W, threads=None):
    """Backward w.r.t. the input, Algorithm 1 line 11: dL/dI = dL/dO x W^T.

    M = tokens, N = in features, K = out features.  With the cached W ([in,out] = [N,K])
    the mode is NT.
    """
    return gemm(M, N, K, layout, dY, W, threads)


def linear_bwd_weight(M, N, K, layout, X, dY, threads=None):
    """Backward w.r.t. the weight, Algorithm 1 line 13: dL/dW = I^T x dL/dO.

    M = in features, N = out features, K = tokens.  With the cached I ([tokens,in] = [K,M])
    and dL/dO ([tokens,out] = [K,N]) the mode is TN.
    """
    return gemm(M, N, K, layout, X, dY, threads)


def transpose(bits: np.ndarray) -> np.ndarray:
    """The operand re-stored for another mode (Sec. IV-C): [rows, cols] -> [cols, rows], bit patterns moved."""
    if not isinstance(bits, np.ndarray) or bits.dtype != np.uint16 or bits.ndim != 2:
        raise TypeError("expected a 2-D numpy uint16 array of bf16 bit patterns")
    src = np.ascontiguousarray(bits)
    rows, cols = src.shape
    dst = np.empty((cols, rows), dtype=np.uint16)
    rc = _load().oracle_transpose_u16(rows, cols, src.ctypes.data, dst.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_transpose_u16 failed ({rc})")
    return dst
