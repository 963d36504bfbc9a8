"""Drives the CPU emulation of the library (tests/emu): the product's host code and kernel
template run on a functional model of the hardware, with bounds checks and adversarial timing.
The Python binding is reused as it is; only the shared library behind it is swapped for the
duration of a call, and operands are CPU tensors."""
from __future__ import annotations

import contextlib
import ctypes
import importlib.util
import os

import paper_2210_16691_amd as al

HERE = os.path.dirname(os.path.abspath(__file__))

# (late_landing, last_wave_first): when direct-to-LDS data arrives, and which wave runs ahead
POLICIES = [(1, 0), (0, 1), (1, 1), (0, 0)]

_emu = None


def lib() -> ctypes.CDLL:
    global _emu
    if _emu is None:
        import shutil
        import pytest
        if not (os.path.exists("/opt/rocm/llvm/bin/clang++") or shutil.which(os.environ.get("ALCOP_HOST_CXX", ""))):
            pytest.skip("no host clang++ with vector extensions to build the emulation")
        spec = importlib.util.spec_from_file_location("build_emu", os.path.join(HERE, "emu", "build_emu.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        L = al._declare(ctypes.CDLL(mod.build()))
        L.emu_reset.argtypes = [ctypes.c_int, ctypes.c_int]
        L.emu_set_mutation.argtypes = [ctypes.c_int]
        L.emu_register_buffer.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
        L.emu_error_count.restype = ctypes.c_long
        L.emu_error_text.argtypes = [ctypes.c_char_p, ctypes.c_size_t]
        for f in (L.emu_f32_to_f16, L.emu_f32_to_bf16):
            f.argtypes = [ctypes.c_float]
            f.restype = ctypes.c_uint16
        L.emu_f16_to_f32.argtypes = [ctypes.c_uint16]
        L.emu_f16_to_f32.restype = ctypes.c_float
        _emu = L
    return _emu


class NullStream:
    """Stands in for a HIP stream: the emulated launch is synchronous."""
    cuda_stream = 0


def _span_bytes(t) -> int:
    """Bytes from the first to one past the last element a (possibly strided) tensor addresses."""
    if t.numel() == 0:
        return 0
    last = sum((n - 1) * s for n, s in zip(t.shape, t.stride()))
    return (last + 1) * t.element_size()


@contextlib.contextmanager
def _swapped():
    real = al._lib
    al._lib = lib()
    try:
        yield
    finally:
        al._lib = real


def call(fn, *args, reads=(), writes=(), policy=(1, 0), mutation=0, **kw):
    """Runs a binding entry point (al.alcop_gemm, ...) on the emulator.  `reads` / `writes` are the
    tensors the kernel may touch; everything else is out of bounds.  Returns the logged errors."""
    L = lib()
    L.emu_reset(policy[0], policy[1])
    L.emu_set_mutation(mutation)
    for t in reads:
        L.emu_register_buffer(t.data_ptr(), _span_bytes(t), 0)
    for t in writes:
        L.emu_register_buffer(t.data_ptr(), _span_bytes(t), 1)
    with _swapped():
        fn(*args, stream=NullStream(), **kw)
    L.emu_set_mutation(0)
    n = L.emu_error_count()
    if n == 0:
        return []
    buf = ctypes.create_string_buffer(8192)
    L.emu_error_text(buf, 8192)
    return ["%d errors" % n] + buf.value.decode().splitlines()


def space(prob, opt_in=False):
    """Schedules the emulated library holds for a problem (a sample of the product's); with opt_in
    also the kernels outside the default space."""
    with _swapped():
        found = al.alcop_sched_space(prob) + (al.alcop_sched_variants(prob) if opt_in else [])
        return [s for s in found if al.alcop_sched_supported(prob, s) == al.OK]
