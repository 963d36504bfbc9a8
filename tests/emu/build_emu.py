"""Builds the CPU emulation of the library (tests only): the product's host sources plus
emu_lib.cpp, compiled for the host with the clang that ships with ROCm (the kernel header uses
clang vector types), into _build/emu/libalcop_emu.so."""
from __future__ import annotations

import concurrent.futures as cf
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_2210_16691_amd", "csrc")
OUT = os.path.join(ROOT, "_build", "emu")
LIB = os.path.join(OUT, "libalcop_emu.so")
CXX = os.environ.get("ALCOP_HOST_CXX", "/opt/rocm/llvm/bin/clang++")
FLAGS = [os.environ.get("EMU_OPT", "-O1"), "-std=c++17", "-fPIC", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + CSRC,
         "-I" + HERE, "-D__launch_bounds__(...)=", "-Wno-psabi", "-Wno-pass-failed"]


def _newest_dep() -> float:
    deps = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "*.h")) + \
        glob.glob(os.path.join(ROOT, "include", "*.h")) + [os.path.join(HERE, "emu_lib.cpp")]
    return max(os.path.getmtime(d) for d in deps)


def _compile(job) -> str:
    src, obj, extra = job
    if not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), _newest_dep()):
        subprocess.check_call([CXX] + FLAGS + extra + ["-c", src, "-o", obj])
    return obj


def build() -> str:
    os.makedirs(OUT, exist_ok=True)
    emu = os.path.join(HERE, "emu_lib.cpp")
    jobs = [(emu, os.path.join(OUT, "emu_part%d.o" % p), ["-DEMU_PART=%d" % p]) for p in range(8)]
    jobs.append((emu, os.path.join(OUT, "emu_main.o"), ["-DEMU_PART=-1"]))
    for name in ("alcop_api.cpp", "alcop_model.cpp"):
        jobs.append((os.path.join(CSRC, name), os.path.join(OUT, name + ".o"), []))
    with cf.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, jobs))
    if not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        subprocess.check_call([CXX, "-shared", "-o", LIB] + objs +
                              ["-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"])
    return LIB


if __name__ == "__main__":
    print(build())
