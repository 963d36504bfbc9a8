"""ctypes binding of libalcop_diag.so (include/alcop_diag.h): the main loop timed with one class of
operation left out.  A measurement aid; its kernels compute garbage on purpose."""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
FULL, NO_DMA, NO_LDS_READ, NO_MFMA, NO_BARRIER, NO_STORE, NO_SWIZZLE, COPY = 0, 1, 2, 4, 8, 16, 32, 64
EXPORTS = ("alcop_diag_configs", "alcop_diag_config_name", "alcop_diag_time", "alcop_diag_launch_floor")
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        path = os.path.join(HERE, "libalcop_diag.so")
        if not os.path.exists(path):
            raise RuntimeError("libalcop_diag.so is not built: run python -m paper_2210_16691_amd.build")
        L = ctypes.CDLL(path)
        L.alcop_diag_configs.restype = ctypes.c_int
        L.alcop_diag_config_name.restype = ctypes.c_char_p
        L.alcop_diag_config_name.argtypes = [ctypes.c_int]
        L.alcop_diag_time.restype = ctypes.c_int
        L.alcop_diag_time.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.POINTER(ctypes.c_double)]
        L.alcop_diag_launch_floor.restype = ctypes.c_int
        L.alcop_diag_launch_floor.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
        _lib = L
    return _lib


def configs():
    L = lib()
    return [L.alcop_diag_config_name(i).decode() for i in range(L.alcop_diag_configs())]


def alcop_diag_time(config: int, drop: int, A, B, C, iters: int = 200) -> float:
    """Microseconds per launch of configuration `config` without the operations in `drop`.
    A [M, K], B [K, N], C [M, N]: contiguous CUDA tensors (fp16 or bf16 as the configuration says)."""
    M, K = A.shape
    N = B.shape[1]
    if B.shape[0] != K or tuple(C.shape) != (M, N) or not (A.is_contiguous() and B.is_contiguous() and C.is_contiguous()):
        raise ValueError("operand shapes")
    if not (A.is_cuda and B.is_cuda and C.is_cuda) or A.dtype != B.dtype or A.dtype != C.dtype:
        raise ValueError("operands must be CUDA tensors of one 16-bit dtype")
    us = ctypes.c_double()
    rc = lib().alcop_diag_time(config, drop, A.data_ptr(), B.data_ptr(), C.data_ptr(), M, N, K, iters,
                               ctypes.byref(us))
    if rc != 0:
        raise RuntimeError("alcop_diag_time failed (%d)" % rc)
    return us.value


def alcop_diag_launch_floor(blocks: int = 256, threads: int = 256, iters: int = 1000) -> float:
    """Microseconds per launch of an empty kernel of that shape, launches back to back."""
    us = ctypes.c_double()
    rc = lib().alcop_diag_launch_floor(blocks, threads, iters, ctypes.byref(us))
    if rc != 0:
        raise RuntimeError("alcop_diag_launch_floor failed (%d)" % rc)
    return us.value
