"""CPU oracle for the ALCOP hot path (GEMM, batched matmul, conv2d) - TEST INFRASTRUCTURE ONLY.

The arithmetic lives in ``alcop_oracle.c`` (plain C, fp64 accumulation, reduction
index ascending; see that file's header for the definitions and the paper passages
they follow).  This module only compiles that file with gcc, loads it with ctypes
and marshals numpy arrays.  The static performance model of the paper's Sec. 5 is
restated independently in ``oracle/perf_model.py``.

Nothing under the product package imports this module, and this module imports
nothing from the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "alcop_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F16 = 0
BF16 = 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over output rows). Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        i, l = ctypes.c_int, ctypes.c_long
        lib.alcop_oracle_decode_f16.restype = ctypes.c_double
        lib.alcop_oracle_decode_f16.argtypes = [ctypes.c_uint16]
        lib.alcop_oracle_decode_bf16.restype = ctypes.c_double
        lib.alcop_oracle_decode_bf16.argtypes = [ctypes.c_uint16]
        lib.alcop_oracle_decode.restype = None
        lib.alcop_oracle_decode.argtypes = [u16p, f64p, ctypes.c_size_t, i]
        lib.alcop_oracle_threads.restype = i
        lib.alcop_oracle_gemm.restype = i
        lib.alcop_oracle_gemm.argtypes = [u16p, u16p, f64p, i, i, i, l, l, l, i, i, i]
        lib.alcop_oracle_bmm.restype = i
        lib.alcop_oracle_bmm.argtypes = [u16p, u16p, f64p, i, i, i, i, l, l, l, l, l, l, i, i, i]
        lib.alcop_oracle_conv2d.restype = i
        lib.alcop_oracle_conv2d.argtypes = [u16p, u16p, f64p] + [i] * 12
        lib.alcop_oracle_conv2d_dilated.restype = i
        lib.alcop_oracle_conv2d_dilated.argtypes = [u16p, u16p, f64p] + [i] * 14
        _lib = lib
    return _lib


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("oracle inputs are uint16 bit patterns, got %s" % a.dtype)
    return a


def _p16(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _p64(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().alcop_oracle_threads())


def decode(bits, dtype: int) -> np.ndarray:
    """Exact fp64 value of every 16-bit pattern in ``bits`` (binary16 or bfloat16)."""
    b = _u16(bits)
    out = np.empty(b.shape, dtype=np.float64)
    _load().alcop_oracle_decode(_p16(b), _p64(out), b.size, dtype)
    return out


def gemm(A, B, dtype: int, transA: bool = False, transB: bool = False) -> np.ndarray:
    """C = A.B in fp64.  A is MxK (or KxM if transA), B is KxN (or NxK if transB); 2-D uint16."""
    A, B = _u16(A), _u16(B)
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    K2, N = (B.shape[1], B.shape[0]) if transB else B.shape
    if K != K2:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, K2))
    C = np.empty((M, N), dtype=np.float64)
    rc = _load().alcop_oracle_gemm(_p16(A), _p16(B), _p64(C), M, N, K,
                                   A.shape[1], B.shape[1], N, int(transA), int(transB), dtype)
    if rc:
        raise MemoryError("oracle gemm failed (%d)" % rc)
    return C


def bmm(A, B, dtype: int, transA: bool = False, transB: bool = False) -> np.ndarray:
    """Batched C[b] = A[b].B[b] in fp64; A, B are 3-D uint16 with the batch index first."""
    A, B = _u16(A), _u16(B)
    batch = A.shape[0]
    if B.shape[0] != batch:
        raise ValueError("batch sizes differ")
    M, K = (A.shape[2], A.shape[1]) if transA else A.shape[1:]
    K2, N = (B.shape[2], B.shape[1]) if transB else B.shape[1:]
    if K != K2:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, K2))
    C = np.empty((batch, M, N), dtype=np.float64)
    rc = _load().alcop_oracle_bmm(_p16(A), _p16(B), _p64(C), batch, M, N, K,
                                  A.shape[2], B.shape[2], N,
                                  A.shape[1] * A.shape[2], B.shape[1] * B.shape[2], M * N,
                                  int(transA), int(transB), dtype)
    if rc:
        raise MemoryError("oracle bmm failed (%d)" % rc)
    return C


def conv2d(x, w, dtype: int, stride=(1, 1), pad=(0, 0), dilation=(1, 1)) -> np.ndarray:
    """y[n,p,q,k] = sum_{r,s,c} x[n, p*sh-ph+r*dh, q*sw-pw+s*dw, c] * w[r,s,c,k] in fp64 (zero padding).
    Dilation (1, 1) is the paper's operator and runs the plain seven-loop routine; any other
    dilation runs the routine that carries the two extra factors."""
    x, w = _u16(x), _u16(w)
    N, H, W, C = x.shape
    R, S, C2, K = w.shape
    if C != C2:
        raise ValueError("channel counts differ")
    sh, sw = stride
    ph, pw = pad
    dh, dw = dilation
    P = (H + 2 * ph - dh * (R - 1) - 1) // sh + 1
    Q = (W + 2 * pw - dw * (S - 1) - 1) // sw + 1
    y = np.empty((N, P, Q, K), dtype=np.float64)
    if (dh, dw) == (1, 1):
        rc = _load().alcop_oracle_conv2d(_p16(x), _p16(w), _p64(y), N, H, W, C, K, R, S,
                                         sh, sw, ph, pw, dtype)
    else:
        rc = _load().alcop_oracle_conv2d_dilated(_p16(x), _p16(w), _p64(y), N, H, W, C, K, R, S,
                                                 sh, sw, ph, pw, dh, dw, dtype)
    if rc:
        raise MemoryError("oracle conv2d failed (%d)" % rc)
    return y


def epilogue(C: np.ndarray, alpha: float = 1.0, bias=None, act: int = 0) -> np.ndarray:
    """Elementwise function fused on the consumer side (paper Sec. 3.2):
    act(alpha * C[..., j] + bias[j]) in fp64; act 0 = identity, 1 = ReLU."""
    out = np.asarray(C, dtype=np.float64) * float(alpha)
    if bias is not None:
        out = out + np.asarray(bias, dtype=np.float64)
    if act == 1:
        out = np.where(out < 0.0, 0.0, out)
    return out
