"""MI355X-native load-compute-pipelined GEMM / BMM / implicit-GEMM conv2d (ALCOP, arXiv 2210.16691).

Thin ctypes binding over ``libalcop.so`` (C ABI declared in ``include/alcop.h``).  Argument
marshalling only: every step of the hot path runs in the HIP kernels.  PyTorch is used for device
memory and streams.  There is no CPU fallback: if the shared library is missing, importing the
binding's functions raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libalcop.so")

F16, BF16, F32 = 0, 1, 2
OP_GEMM, OP_BMM, OP_CONV2D = 0, 1, 2

OK = 0
ERR_NULL, ERR_DTYPE, ERR_ALIGN, ERR_SHAPE, ERR_SCHED, ERR_LAUNCH, ERR_UNSUPPORTED, ERR_SIZE, ERR_IO = (
    -1, -2, -3, -4, -5, -6, -7, -8, -9)

EXPORTS = [
    "alcop_gemm", "alcop_bmm", "alcop_gemm_fused", "alcop_bmm_fused", "alcop_conv2d_igemm", "alcop_sched_supported", "alcop_sched_space",
    "alcop_model_predict", "alcop_tune", "alcop_time", "alcop_strerror", "alcop_version",
    "alcop_sched_auto", "alcop_cache_save", "alcop_cache_load",
    "alcop_corrector_features", "alcop_corrector_fit", "alcop_splitk_workspace_bytes", "alcop_gemm_splitk", "alcop_gemm_splitk_static", "alcop_conv2d_igemm_splitk", "alcop_splitk_auto", "alcop_splitk_space", "alcop_tune_splitk", "alcop_conv2d_igemm_krsc", "alcop_conv2d_igemm_fused", "alcop_conv2d_igemm_dilated", "alcop_sched_variants", "alcop_sched_ranked",
    "alcop_unaligned_workspace_bytes", "alcop_bmm_unaligned", "alcop_conv2d_unaligned_workspace_bytes",
    "alcop_conv2d_igemm_unaligned", "alcop_init",
]


class AlcopError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__("%s failed: %s (%d)" % (what, strerror(code), code))
        self.code = code


class Sched(ctypes.Structure):
    """Mirror of ``alcop_sched``."""
    _fields_ = [(n, ctypes.c_int) for n in
                ("bm", "bn", "bk", "wm", "wn", "stages", "reg_stages", "fuse_inner", "raster",
                 "l2_prefetch", "variant")]

    def key(self):
        return tuple(getattr(self, n) for n, _ in self._fields_)

    def __repr__(self):
        return "Sched(%dx%dx%d w%dx%d S%d R%d F%d r%d pf%d)" % self.key()[:10] + (
            "" if self.variant == 0 else "[v%d]" % self.variant)


def sched(bm, bn, bk, wm, wn, stages=1, reg_stages=1, fuse_inner=0, raster=1, l2_prefetch=0,
          variant=0) -> Sched:
    return Sched(bm, bn, bk, wm, wn, stages, reg_stages, fuse_inner, raster, l2_prefetch, variant)


class Epilogue(ctypes.Structure):
    """Mirror of ``alcop_epilogue``: C = act(alpha * A.B + bias[j])."""
    _fields_ = [("alpha", ctypes.c_float), ("bias", ctypes.c_void_p), ("act", ctypes.c_int)]


class Problem(ctypes.Structure):
    """Mirror of ``alcop_problem``."""
    _fields_ = [("op", ctypes.c_int), ("batch", ctypes.c_int), ("M", ctypes.c_int),
                ("N", ctypes.c_int), ("K", ctypes.c_int), ("transB", ctypes.c_int),
                ("in_", ctypes.c_int), ("out", ctypes.c_int), ("conv_C", ctypes.c_int),
                ("transA", ctypes.c_int)]


_lib = None


def _declare(L: ctypes.CDLL) -> ctypes.CDLL:
    """Sets the argument and result types of every entry point of include/alcop.h on L."""
    vp, i, l = ctypes.c_void_p, ctypes.c_int, ctypes.c_long
    dp = ctypes.POINTER(ctypes.c_double)
    ip = ctypes.POINTER(ctypes.c_int)
    sp = ctypes.POINTER(Sched)
    pp = ctypes.POINTER(Problem)
    ep = ctypes.POINTER(Epilogue)
    L.alcop_gemm.restype = i
    L.alcop_gemm.argtypes = [vp, vp, vp, i, i, i, l, l, l, i, i, i, i, sp, vp]
    L.alcop_bmm.restype = i
    L.alcop_bmm.argtypes = [vp, vp, vp, i, i, i, i, l, l, l, l, l, l, i, i, i, i, sp, vp]
    L.alcop_gemm_fused.restype = i
    L.alcop_gemm_fused.argtypes = [vp, vp, vp, i, i, i, l, l, l, i, i, i, i, ep, sp, vp]
    L.alcop_bmm_fused.restype = i
    L.alcop_bmm_fused.argtypes = [vp, vp, vp, i, i, i, i, l, l, l, l, l, l, i, i, i, i, ep, sp, vp]
    L.alcop_conv2d_igemm.restype = i
    L.alcop_conv2d_igemm.argtypes = [vp, vp, vp] + [i] * 11 + [i, i, sp, vp]
    L.alcop_conv2d_igemm_krsc.restype = i
    L.alcop_conv2d_igemm_krsc.argtypes = [vp, vp, vp] + [i] * 11 + [i, i, sp, vp]
    L.alcop_conv2d_igemm_fused.restype = i
    L.alcop_conv2d_igemm_fused.argtypes = [vp, vp, vp] + [i] * 11 + [i, i, ep, i, sp, vp]
    L.alcop_sched_supported.restype = i
    L.alcop_sched_supported.argtypes = [pp, sp]
    L.alcop_sched_space.restype = i
    L.alcop_sched_space.argtypes = [pp, sp, i]
    L.alcop_model_predict.restype = i
    L.alcop_model_predict.argtypes = [pp, sp, i, dp, dp]
    L.alcop_tune.restype = i
    L.alcop_tune.argtypes = [pp, vp, vp, vp, l, l, l, l, l, l, ip, i, i, i, i, sp, dp, ip, ip,
                             sp, dp, dp, i, vp]
    L.alcop_sched_ranked.restype = i
    L.alcop_sched_ranked.argtypes = [pp, i, i, i, sp, i]
    L.alcop_sched_variants.restype = i
    L.alcop_sched_variants.argtypes = [pp, sp, i]
    L.alcop_time.restype = i
    L.alcop_time.argtypes = [pp, vp, vp, vp, l, l, l, l, l, l, ip, sp, i, i, dp, vp]
    L.alcop_sched_auto.restype = i
    L.alcop_sched_auto.argtypes = [pp, sp]
    L.alcop_cache_save.restype = i
    L.alcop_cache_save.argtypes = [ctypes.c_char_p]
    L.alcop_cache_load.restype = i
    L.alcop_cache_load.argtypes = [ctypes.c_char_p]
    L.alcop_corrector_features.restype = i
    L.alcop_corrector_features.argtypes = [pp, sp, dp]
    L.alcop_corrector_fit.restype = i
    L.alcop_corrector_fit.argtypes = [dp, dp, i, dp]
    sz = ctypes.c_size_t
    L.alcop_splitk_workspace_bytes.restype = sz
    L.alcop_splitk_workspace_bytes.argtypes = [i, i, i, i]
    L.alcop_gemm_splitk.restype = i
    L.alcop_gemm_splitk.argtypes = [vp, vp, vp, i, i, i, i, l, l, l, l, l, l, i, i, i, i, ep, sp, i,
                                    vp, sz, vp]
    L.alcop_gemm_splitk_static.restype = i
    L.alcop_gemm_splitk_static.argtypes = [vp, vp, vp, i, i, i, i, l, l, l, l, l, l, i, i, i, i, ep, sp, i, vp]
    L.alcop_conv2d_igemm_dilated.restype = i
    L.alcop_conv2d_igemm_dilated.argtypes = [vp, vp, vp] + [i] * 14 + [i, i, ep, sp, vp]
    L.alcop_unaligned_workspace_bytes.restype = sz
    L.alcop_unaligned_workspace_bytes.argtypes = [i, i, i, i, i]
    L.alcop_bmm_unaligned.restype = i
    L.alcop_bmm_unaligned.argtypes = [vp, vp, vp, i, i, i, i, l, l, l, l, l, l, i, i, i, i, ep, sp, vp, sz, vp]
    L.alcop_conv2d_unaligned_workspace_bytes.restype = sz
    L.alcop_conv2d_unaligned_workspace_bytes.argtypes = [i] * 14
    L.alcop_conv2d_igemm_unaligned.restype = i
    L.alcop_conv2d_igemm_unaligned.argtypes = [vp, vp, vp] + [i] * 13 + [i, i, ep, sp, vp, sz, vp]
    L.alcop_conv2d_igemm_splitk.restype = i
    L.alcop_conv2d_igemm_splitk.argtypes = [vp, vp, vp] + [i] * 11 + [i, i, sp, i, vp, sz, vp]
    L.alcop_tune_splitk.restype = i
    L.alcop_tune_splitk.argtypes = [pp, vp, vp, vp, l, l, l, l, l, l, ip, vp, sz, i, i, sp, ip, dp, ip, ip,
                                    sp, ip, dp, dp, i, vp]
    L.alcop_splitk_space.restype = i
    L.alcop_splitk_space.argtypes = [pp, sp, i]
    L.alcop_splitk_auto.restype = i
    L.alcop_splitk_auto.argtypes = [pp, i, sp, ip, dp]
    L.alcop_init.restype = i
    L.alcop_init.argtypes = []
    L.alcop_strerror.restype = ctypes.c_char_p
    L.alcop_strerror.argtypes = [i]
    L.alcop_version.restype = ctypes.c_char_p
    L.alcop_version.argtypes = []
    return L


def lib() -> ctypes.CDLL:
    """Loads libalcop.so (built by ``python -m paper_2210_16691_amd.build``); fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libalcop.so is not built: run `python -m paper_2210_16691_amd.build`")
        _lib = _declare(ctypes.CDLL(LIB_PATH))
    return _lib


def alcop_init() -> None:
    """Does ahead of time what the first call of each entry point would do besides launching."""
    _check(lib().alcop_init(), "alcop_init")


def strerror(code: int) -> str:
    return lib().alcop_strerror(int(code)).decode()


def version() -> str:
    return lib().alcop_version().decode()


# ---- marshalling helpers ---------------------------------------------------------------------
def _dtype_code(t) -> int:
    import torch
    return {torch.float16: F16, torch.bfloat16: BF16, torch.float32: F32}[t.dtype]


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _sp(s):
    return ctypes.byref(s) if s is not None else None


def _check(rc, what):
    if rc != OK:
        raise AlcopError(rc, what)


def _same_place(*ts):
    dev = ts[0].device
    for t in ts:
        if t is not None and t.device != dev:
            raise ValueError("operands live on different devices: %s and %s" % (dev, t.device))


def _mm_shapes(A, B, C, transA, transB, bias=None):
    """Operand checks of the matrix entry points, before anything reaches the C call: the library
    sizes its buffer descriptors from (M, N, K) and the leading dimensions it is told, so a tensor
    that does not have that shape would be read or written past its end on the GPU.  Returns
    (batch, M, N, K)."""
    if A.dim() != B.dim() or A.dim() != C.dim() or A.dim() not in (2, 3):
        raise ValueError("A, B, C must all be 2-D (GEMM) or all 3-D (batched)")
    if A.dtype != B.dtype:
        raise ValueError("A and B differ in dtype: %s and %s" % (A.dtype, B.dtype))
    _dtype_code(C)
    _same_place(A, B, C, bias)
    for name, t in (("A", A), ("B", B), ("C", C)):
        if t.stride(-1) != 1:
            raise ValueError("%s: the last dimension must be contiguous" % name)
    b = A.shape[0] if A.dim() == 3 else 1
    if A.dim() == 3 and (B.shape[0] != b or C.shape[0] != b):
        raise ValueError("batch sizes differ: %d, %d, %d" % (b, B.shape[0], C.shape[0]))
    K, M = tuple(A.shape[-2:]) if transA else tuple(A.shape[-2:])[::-1]
    Kb, N = tuple(B.shape[-2:])[::-1] if transB else tuple(B.shape[-2:])
    if Kb != K:
        raise ValueError("reduction extents differ: A has K = %d, B has K = %d" % (K, Kb))
    if tuple(C.shape[-2:]) != (M, N):
        raise ValueError("C is %s, expected %s" % (tuple(C.shape[-2:]), (M, N)))
    if bias is not None and (bias.dim() != 1 or bias.shape[0] != N or not bias.is_contiguous()
                             or bias.element_size() != 4 or not bias.is_floating_point()):
        raise ValueError("bias must be a contiguous fp32 vector of N = %d values" % N)
    return b, M, N, K


def _conv_shapes(x, w, y, stride, pad, krsc=False, bias=None, dilation=(1, 1)):
    """Operand checks of the convolution entry points.  Returns (N, H, W, C, K, R, S)."""
    if x.dim() != 4 or w.dim() != 4 or y.dim() != 4:
        raise ValueError("x, w, y must be 4-D (NHWC, RSCK or KRSC, NPQK)")
    if x.dtype != w.dtype:
        raise ValueError("x and w differ in dtype: %s and %s" % (x.dtype, w.dtype))
    _dtype_code(y)
    _same_place(x, w, y, bias)
    for name, t in (("x", x), ("w", w), ("y", y)):
        if not t.is_contiguous():
            raise ValueError("%s must be contiguous" % name)
    N, H, W, Cc = x.shape
    if krsc:
        K, R, S, Cw = w.shape
    else:
        R, S, Cw, K = w.shape
    if Cw != Cc:
        raise ValueError("channel counts differ: x has %d, w has %d" % (Cc, Cw))
    if stride[0] <= 0 or stride[1] <= 0 or pad[0] < 0 or pad[1] < 0 or dilation[0] <= 0 or dilation[1] <= 0:
        raise ValueError("stride and dilation must be positive and padding non-negative")
    P = (H + 2 * pad[0] - dilation[0] * (R - 1) - 1) // stride[0] + 1
    Q = (W + 2 * pad[1] - dilation[1] * (S - 1) - 1) // stride[1] + 1
    if tuple(y.shape) != (N, P, Q, K):
        raise ValueError("y is %s, expected %s" % (tuple(y.shape), (N, P, Q, K)))
    if bias is not None and (bias.dim() != 1 or bias.shape[0] != K or not bias.is_contiguous()
                             or bias.element_size() != 4 or not bias.is_floating_point()):
        raise ValueError("bias must be a contiguous fp32 vector of K = %d values" % K)
    return N, H, W, Cc, K, R, S


# ---- the entry points (same names as the C ABI) ----------------------------------------------
def alcop_gemm(A, B, C, sched=None, transB=False, stream=None, transA=False):
    """C[M,N] = A . B  (A is [M,K], or [K,M] if transA; B is [K,N], or [N,K] if transB).  Tensors
    are 2-D CUDA tensors whose last dimension is contiguous; C's dtype selects the output type."""
    if A.dim() != 2:
        raise ValueError("alcop_gemm takes 2-D tensors")
    _, M, N, K = _mm_shapes(A, B, C, transA, transB)
    rc = lib().alcop_gemm(_ptr(A), _ptr(B), _ptr(C), M, N, K, A.stride(0), B.stride(0), C.stride(0),
                          int(transA), int(transB), _dtype_code(A), _dtype_code(C), _sp(sched),
                          _stream(stream))
    _check(rc, "alcop_gemm")
    return C


def alcop_bmm(A, B, C, sched=None, transB=False, stream=None, transA=False):
    """Batched: A [b,M,K] (or [b,K,M] if transA), B [b,K,N] (or [b,N,K] if transB), C [b,M,N]."""
    if A.dim() != 3:
        raise ValueError("alcop_bmm takes 3-D tensors")
    b, M, N, K = _mm_shapes(A, B, C, transA, transB)
    rc = lib().alcop_bmm(_ptr(A), _ptr(B), _ptr(C), b, M, N, K, A.stride(1), B.stride(1), C.stride(1),
                         A.stride(0), B.stride(0), C.stride(0), int(transA), int(transB),
                         _dtype_code(A), _dtype_code(C), _sp(sched), _stream(stream))
    _check(rc, "alcop_bmm")
    return C


def _epilogue(alpha, bias, act):
    return Epilogue(float(alpha), bias.data_ptr() if bias is not None else None, int(act))


def alcop_gemm_fused(A, B, C, alpha=1.0, bias=None, act=0, sched=None, transB=False, stream=None):
    """C = act(alpha * A.B + bias[j]); bias is an fp32 CUDA vector of N values or None; act 1 = ReLU."""
    if A.dim() != 2:
        raise ValueError("alcop_gemm_fused takes 2-D tensors")
    _, M, N, K = _mm_shapes(A, B, C, False, transB, bias)
    e = _epilogue(alpha, bias, act)
    rc = lib().alcop_gemm_fused(_ptr(A), _ptr(B), _ptr(C), M, N, K, A.stride(0), B.stride(0),
                                C.stride(0), 0, int(transB), _dtype_code(A), _dtype_code(C),
                                ctypes.byref(e), _sp(sched), _stream(stream))
    _check(rc, "alcop_gemm_fused")
    return C


def alcop_bmm_fused(A, B, C, alpha=1.0, bias=None, act=0, sched=None, transB=False, stream=None):
    if A.dim() != 3:
        raise ValueError("alcop_bmm_fused takes 3-D tensors")
    b, M, N, K = _mm_shapes(A, B, C, False, transB, bias)
    e = _epilogue(alpha, bias, act)
    rc = lib().alcop_bmm_fused(_ptr(A), _ptr(B), _ptr(C), b, M, N, K, A.stride(1), B.stride(1),
                               C.stride(1), A.stride(0), B.stride(0), C.stride(0), 0, int(transB),
                               _dtype_code(A), _dtype_code(C), ctypes.byref(e), _sp(sched),
                               _stream(stream))
    _check(rc, "alcop_bmm_fused")
    return C


def alcop_conv2d_igemm(x, w, y, stride=(1, 1), pad=(0, 0), sched=None, stream=None):
    """x NHWC [N,H,W,C], w RSCK [R,S,C,K], y NPQK [N,P,Q,K]; all contiguous."""
    N, H, W, Cc, K, R, S = _conv_shapes(x, w, y, stride, pad)
    rc = lib().alcop_conv2d_igemm(_ptr(x), _ptr(w), _ptr(y), N, H, W, Cc, K, R, S,
                                  stride[0], stride[1], pad[0], pad[1],
                                  _dtype_code(x), _dtype_code(y), _sp(sched), _stream(stream))
    _check(rc, "alcop_conv2d_igemm")
    return y


def alcop_splitk_workspace_bytes(batch: int, M: int, N: int, split: int) -> int:
    return int(lib().alcop_splitk_workspace_bytes(batch, M, N, split))


def alcop_gemm_splitk(A, B, C, split, workspace, sched=None, alpha=1.0, bias=None, act=0,
                      transB=False, stream=None, transA=False):
    """C = act(alpha * A.B + bias) with the reduction axis cut into `split` slices (0 = the model's
    choice).  A, B, C are 2-D (GEMM) or 3-D (batched) tensors; `workspace` is a tensor of at least
    alcop_splitk_workspace_bytes(batch, M, N, split) bytes that the call overwrites."""
    b, M, N, K = _mm_shapes(A, B, C, transA, transB, bias)
    if A.dim() == 2:
        sA, sB, sC = 0, 0, 0
        lda, ldb, ldc = A.stride(0), B.stride(0), C.stride(0)
    else:
        lda, ldb, ldc = A.stride(1), B.stride(1), C.stride(1)
        sA, sB, sC = A.stride(0), B.stride(0), C.stride(0)
    e = _epilogue(alpha, bias, act)
    rc = lib().alcop_gemm_splitk(_ptr(A), _ptr(B), _ptr(C), b, M, N, K, lda, ldb, ldc, sA, sB, sC,
                                 int(transA), int(transB), _dtype_code(A), _dtype_code(C),
                                 ctypes.byref(e), _sp(sched), int(split), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "alcop_gemm_splitk")
    return C


SPLITK_STATIC_BYTES = 32 << 20


def alcop_gemm_splitk_static(A, B, C, split, sched=None, alpha=1.0, bias=None, act=0,
                             transB=False, stream=None, transA=False):
    """alcop_gemm_splitk without a workspace argument: the partial tiles go to the library's own
    device array (at most SPLITK_STATIC_BYTES); the call allocates nothing."""
    b, M, N, K = _mm_shapes(A, B, C, transA, transB, bias)
    if A.dim() == 2:
        sA, sB, sC = 0, 0, 0
        lda, ldb, ldc = A.stride(0), B.stride(0), C.stride(0)
    else:
        lda, ldb, ldc = A.stride(1), B.stride(1), C.stride(1)
        sA, sB, sC = A.stride(0), B.stride(0), C.stride(0)
    e = _epilogue(alpha, bias, act)
    rc = lib().alcop_gemm_splitk_static(_ptr(A), _ptr(B), _ptr(C), b, M, N, K, lda, ldb, ldc, sA, sB,
                                        sC, int(transA), int(transB), _dtype_code(A), _dtype_code(C),
                                        ctypes.byref(e), _sp(sched), int(split), _stream(stream))
    _check(rc, "alcop_gemm_splitk_static")
    return C


def alcop_conv2d_igemm_splitk(x, w, y, split, workspace, stride=(1, 1), pad=(0, 0), sched=None,
                              stream=None):
    """alcop_conv2d_igemm with the reduction axis R*S*C cut into `split` slices."""
    N, H, W, Cc, K, R, S = _conv_shapes(x, w, y, stride, pad)
    _same_place(x, workspace)
    rc = lib().alcop_conv2d_igemm_splitk(_ptr(x), _ptr(w), _ptr(y), N, H, W, Cc, K, R, S,
                                         stride[0], stride[1], pad[0], pad[1],
                                         _dtype_code(x), _dtype_code(y), _sp(sched), int(split),
                                         _ptr(workspace), workspace.numel() * workspace.element_size(),
                                         _stream(stream))
    _check(rc, "alcop_conv2d_igemm_splitk")
    return y


def alcop_splitk_space(prob: "Problem"):
    n = lib().alcop_splitk_space(ctypes.byref(prob), None, 0)
    if n < 0:
        raise AlcopError(n, "alcop_splitk_space")
    arr = (Sched * max(n, 1))()
    lib().alcop_splitk_space(ctypes.byref(prob), arr, n)
    return [Sched(*arr[i].key()) for i in range(n)]


def alcop_splitk_auto(prob: "Problem", split: int = 0):
    """Returns (schedule, split, predicted_us): the model's pick among the split-K variants."""
    s, n, us = Sched(), ctypes.c_int(), ctypes.c_double()
    _check(lib().alcop_splitk_auto(ctypes.byref(prob), int(split), ctypes.byref(s), ctypes.byref(n),
                                   ctypes.byref(us)), "alcop_splitk_auto")
    return s, n.value, us.value


def alcop_conv2d_igemm_fused(x, w, y, stride=(1, 1), pad=(0, 0), alpha=1.0, bias=None, act=0,
                             krsc=False, sched=None, stream=None):
    """y = act(alpha * conv(x, w) + bias[k]); w is RSCK [R,S,C,K], or KRSC [K,R,S,C] if krsc."""
    N, H, W, Cc, K, R, S = _conv_shapes(x, w, y, stride, pad, krsc, bias)
    e = _epilogue(alpha, bias, act)
    rc = lib().alcop_conv2d_igemm_fused(_ptr(x), _ptr(w), _ptr(y), N, H, W, Cc, K, R, S,
                                        stride[0], stride[1], pad[0], pad[1], _dtype_code(x),
                                        _dtype_code(y), ctypes.byref(e), int(krsc), _sp(sched),
                                        _stream(stream))
    _check(rc, "alcop_conv2d_igemm_fused")
    return y


def alcop_conv2d_igemm_dilated(x, w, y, stride=(1, 1), pad=(0, 0), dilation=(1, 1), alpha=1.0, bias=None,
                               act=0, krsc=False, sched=None, stream=None):
    """y = act(alpha * conv(x, w) + bias[k]) with filter taps dilation[0] rows / dilation[1] columns
    apart; w is RSCK [R,S,C,K], or KRSC [K,R,S,C] if krsc."""
    N, H, W, Cc, K, R, S = _conv_shapes(x, w, y, stride, pad, krsc, bias, dilation)
    e = _epilogue(alpha, bias, act)
    rc = lib().alcop_conv2d_igemm_dilated(_ptr(x), _ptr(w), _ptr(y), N, H, W, Cc, K, R, S,
                                          stride[0], stride[1], pad[0], pad[1], dilation[0], dilation[1],
                                          int(krsc), _dtype_code(x), _dtype_code(y), ctypes.byref(e),
                                          _sp(sched), _stream(stream))
    _check(rc, "alcop_conv2d_igemm_dilated")
    return y


def alcop_unaligned_workspace_bytes(batch, M, N, K, out_dtype) -> int:
    return lib().alcop_unaligned_workspace_bytes(batch, M, N, K, out_dtype)


def alcop_bmm_unaligned(A, B, C, workspace, alpha=1.0, bias=None, act=0, sched=None, transA=False,
                        transB=False, stream=None):
    """C = act(alpha * A.B + bias[j]) for operands of any extent and element-aligned placement
    (2-D: a GEMM; 3-D: batched); they are padded into `workspace` (a CUDA byte tensor of at least
    alcop_unaligned_workspace_bytes(...) bytes) and multiplied there."""
    b, M, N, K = _mm_shapes(A, B, C, transA, transB, bias)
    _same_place(A, workspace)
    if not workspace.is_contiguous():
        raise ValueError("workspace must be contiguous")
    e = _epilogue(alpha, bias, act)
    if A.dim() == 3:
        ld = (A.stride(1), B.stride(1), C.stride(1), A.stride(0), B.stride(0), C.stride(0))
    else:
        ld = (A.stride(0), B.stride(0), C.stride(0), 0, 0, 0)
    rc = lib().alcop_bmm_unaligned(_ptr(A), _ptr(B), _ptr(C), b, M, N, K, *ld, int(transA), int(transB),
                                   _dtype_code(A), _dtype_code(C), ctypes.byref(e), _sp(sched),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream(stream))
    _check(rc, "alcop_bmm_unaligned")
    return C


def alcop_conv2d_unaligned_workspace_bytes(N, H, W, C, K, R, S, stride, pad, dilation, out_dtype) -> int:
    return lib().alcop_conv2d_unaligned_workspace_bytes(N, H, W, C, K, R, S, stride[0], stride[1], pad[0],
                                                        pad[1], dilation[0], dilation[1], out_dtype)


def alcop_conv2d_igemm_unaligned(x, w, y, workspace, stride=(1, 1), pad=(0, 0), dilation=(1, 1), alpha=1.0,
                                 bias=None, act=0, sched=None, stream=None):
    """y = act(alpha * conv(x, w) + bias[k]) for any channel counts (x NHWC, w RSCK, y NPQK); the
    tensors are padded to 8 channels in `workspace` and convolved there."""
    N, H, W, Cc, K, R, S = _conv_shapes(x, w, y, stride, pad, False, bias, dilation)
    _same_place(x, workspace)
    if not workspace.is_contiguous():
        raise ValueError("workspace must be contiguous")
    e = _epilogue(alpha, bias, act)
    rc = lib().alcop_conv2d_igemm_unaligned(_ptr(x), _ptr(w), _ptr(y), N, H, W, Cc, K, R, S, stride[0],
                                            stride[1], pad[0], pad[1], dilation[0], dilation[1],
                                            _dtype_code(x), _dtype_code(y), ctypes.byref(e), _sp(sched),
                                            _ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _stream(stream))
    _check(rc, "alcop_conv2d_igemm_unaligned")
    return y


def alcop_conv2d_igemm_krsc(x, w, y, stride=(1, 1), pad=(0, 0), sched=None, stream=None):
    """x NHWC [N,H,W,C], w KRSC [K,R,S,C], y NPQK [N,P,Q,K]; all contiguous."""
    N, H, W, Cc, K, R, S = _conv_shapes(x, w, y, stride, pad, krsc=True)
    rc = lib().alcop_conv2d_igemm_krsc(_ptr(x), _ptr(w), _ptr(y), N, H, W, Cc, K, R, S,
                                       stride[0], stride[1], pad[0], pad[1],
                                       _dtype_code(x), _dtype_code(y), _sp(sched), _stream(stream))
    _check(rc, "alcop_conv2d_igemm_krsc")
    return y


def problem(op, M, N, K, in_dtype, out_dtype, batch=1, transB=False, conv_C=0, transA=False) -> Problem:
    return Problem(op, batch, M, N, K, int(transB), in_dtype, out_dtype, conv_C, int(transA))


def alcop_sched_supported(prob: Problem, s: Sched) -> int:
    return lib().alcop_sched_supported(ctypes.byref(prob), ctypes.byref(s))


def alcop_sched_space(prob: Problem):
    n = lib().alcop_sched_space(ctypes.byref(prob), None, 0)
    if n < 0:
        raise AlcopError(n, "alcop_sched_space")
    arr = (Sched * max(n, 1))()
    lib().alcop_sched_space(ctypes.byref(prob), arr, n)
    return [Sched(*arr[i].key()) for i in range(n)]


def alcop_sched_variants(prob: Problem):
    """Schedule variants whose feasibility depends on the call (see alcop_sched.variant)."""
    n = lib().alcop_sched_variants(ctypes.byref(prob), None, 0)
    if n < 0:
        raise AlcopError(n, "alcop_sched_variants")
    arr = (Sched * max(n, 1))()
    lib().alcop_sched_variants(ctypes.byref(prob), arr, n)
    return [Sched(*arr[i].key()) for i in range(n)]


def alcop_sched_ranked(prob: Problem, model: int = 0, variants: bool = False, top_k: int = 10):
    """Schedules in the order alcop_tune(top_k, model) would try them."""
    n = lib().alcop_sched_ranked(ctypes.byref(prob), model, int(variants), top_k, None, 0)
    if n < 0:
        raise AlcopError(n, "alcop_sched_ranked")
    arr = (Sched * max(n, 1))()
    lib().alcop_sched_ranked(ctypes.byref(prob), model, int(variants), top_k, arr, n)
    return [Sched(*arr[i].key()) for i in range(n)]


def alcop_sched_auto(prob: Problem) -> Sched:
    """The schedule a None schedule resolves to (tuning cache, else the model's top-1)."""
    s = Sched()
    _check(lib().alcop_sched_auto(ctypes.byref(prob), ctypes.byref(s)), "alcop_sched_auto")
    return s


def alcop_cache_save(path: str) -> int:
    n = lib().alcop_cache_save(os.fsencode(path))
    if n < 0:
        raise AlcopError(n, "alcop_cache_save")
    return n


def alcop_cache_load(path: str) -> int:
    n = lib().alcop_cache_load(os.fsencode(path))
    if n < 0:
        raise AlcopError(n, "alcop_cache_load")
    return n


def alcop_model_predict(prob: Problem, s: Sched, model: int = 0):
    """Returns (predicted_us, terms[8])."""
    us = ctypes.c_double()
    terms = (ctypes.c_double * 8)()
    rc = lib().alcop_model_predict(ctypes.byref(prob), ctypes.byref(s), model, ctypes.byref(us), terms)
    _check(rc, "alcop_model_predict")
    return us.value, list(terms)


CORRECTOR_DIM = 10


def alcop_corrector_features(prob: Problem, s: Sched):
    """Features of a (problem, schedule) pair as the learner of alcop_tune(model=2) sees them."""
    x = (ctypes.c_double * CORRECTOR_DIM)()
    _check(lib().alcop_corrector_features(ctypes.byref(prob), ctypes.byref(s), x), "alcop_corrector_features")
    return list(x)


def alcop_corrector_fit(X, measured_us):
    """Weights of the learner after the given trials (X: rows of CORRECTOR_DIM features)."""
    n = len(measured_us)
    flat = (ctypes.c_double * (n * CORRECTOR_DIM))(*[float(v) for row in X for v in row])
    ys = (ctypes.c_double * max(n, 1))(*[float(v) for v in measured_us])
    w = (ctypes.c_double * CORRECTOR_DIM)()
    _check(lib().alcop_corrector_fit(flat, ys, n, w), "alcop_corrector_fit")
    return list(w)


@dataclass
class TuneResult:
    best: Sched
    best_us: float
    trials: int
    space: int
    log: list   # [(Sched, predicted_us, measured_us)] in rank order


def _operands(prob, A, B, C, conv):
    if prob.op == OP_CONV2D:
        cv = (ctypes.c_int * 11)(*conv)
        return cv, (0, 0, 0, 0, 0, 0)
    if prob.op == OP_BMM:
        return None, (A.stride(1), B.stride(1), C.stride(1), A.stride(0), B.stride(0), C.stride(0))
    return None, (A.stride(0), B.stride(0), C.stride(0), 0, 0, 0)


def alcop_tune(prob: Problem, A, B, C, top_k=10, model=0, iters=20, conv=None, stream=None,
               variants=False) -> TuneResult:
    """Model-ranked tuning on the caller's tensors (C is overwritten). top_k=0: exhaustive.
    variants=True also considers the schedule variants that depend on the call's geometry."""
    cv, ld = _operands(prob, A, B, C, conv)
    cap = max(1, lib().alcop_sched_space(ctypes.byref(prob), None, 0) +
              lib().alcop_sched_variants(ctypes.byref(prob), None, 0))
    best, best_us = Sched(), ctypes.c_double()
    trials, space = ctypes.c_int(), ctypes.c_int()
    ls, lp, lm = (Sched * cap)(), (ctypes.c_double * cap)(), (ctypes.c_double * cap)()
    rc = lib().alcop_tune(ctypes.byref(prob), _ptr(A), _ptr(B), _ptr(C), *ld, cv, top_k, model,
                          int(variants), iters,
                          ctypes.byref(best), ctypes.byref(best_us), ctypes.byref(trials),
                          ctypes.byref(space), ls, lp, lm, cap, _stream(stream))
    _check(rc, "alcop_tune")
    log = [(Sched(*ls[i].key()), lp[i], lm[i]) for i in range(trials.value)]
    return TuneResult(Sched(*best.key()), best_us.value, trials.value, space.value, log)


def alcop_tune_splitk(prob: Problem, A, B, C, workspace, top_k=10, iters=20, conv=None, stream=None):
    """Model-ranked tuning over (split-K variant, slices).  Returns (TuneResult, best_split); the
    log entries are (Sched, slices, predicted_us, measured_us)."""
    cv, ld = _operands(prob, A, B, C, conv)
    cap = 16 * max(1, lib().alcop_splitk_space(ctypes.byref(prob), None, 0))
    best, best_us, best_split = Sched(), ctypes.c_double(), ctypes.c_int()
    trials, space = ctypes.c_int(), ctypes.c_int()
    ls, lk = (Sched * cap)(), (ctypes.c_int * cap)()
    lp, lm = (ctypes.c_double * cap)(), (ctypes.c_double * cap)()
    rc = lib().alcop_tune_splitk(ctypes.byref(prob), _ptr(A), _ptr(B), _ptr(C), *ld, cv, _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), top_k, iters,
                                 ctypes.byref(best), ctypes.byref(best_split), ctypes.byref(best_us),
                                 ctypes.byref(trials), ctypes.byref(space), ls, lk, lp, lm, cap,
                                 _stream(stream))
    _check(rc, "alcop_tune_splitk")
    log = [(Sched(*ls[i].key()), lk[i], lp[i], lm[i]) for i in range(trials.value)]
    return TuneResult(Sched(*best.key()), best_us.value, trials.value, space.value, log), best_split.value


def alcop_time(prob: Problem, A, B, C, s: Sched, warmup=3, iters=20, conv=None, stream=None) -> float:
    """Mean microseconds per launch of one schedule, timed with HIP events on the stream."""
    cv, ld = _operands(prob, A, B, C, conv)
    us = ctypes.c_double()
    rc = lib().alcop_time(ctypes.byref(prob), _ptr(A), _ptr(B), _ptr(C), *ld, cv, ctypes.byref(s),
                          warmup, iters, ctypes.byref(us), _stream(stream))
    _check(rc, "alcop_time")
    return us.value
