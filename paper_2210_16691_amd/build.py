"""Build step: compiles the HIP sources under csrc/ for gfx950 and links libalcop.so in-tree.

    python -m paper_2210_16691_amd.build [-j N] [--force]

Objects go to _build/ (not committed); the shared library lands beside this file so that it
travels with the source tree.  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
ROOT = os.path.dirname(HERE)
OBJDIR = os.path.join(ROOT, "_build", "alcop")
LIB = os.path.join(HERE, "libalcop.so")
DIAG_LIB = os.path.join(HERE, "libalcop_diag.so")     # measurement aid: csrc/diag_*.hip

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def sources():
    hip = [f for f in glob.glob(os.path.join(CSRC, "*.hip")) if not os.path.basename(f).startswith("diag_")]
    return sorted(hip + glob.glob(os.path.join(CSRC, "*.cpp")))


def diag_sources():
    return sorted(glob.glob(os.path.join(CSRC, "diag_*.hip")))


def _deps_mtime(obj: str) -> float:
    """Newest modification time among the headers this object was last compiled from (from the
    compiler's own dependency file; every header if there is none yet)."""
    dep = obj + ".d"
    if os.path.exists(dep):
        words = open(dep).read().replace("\\\n", " ").split()
        files = [w for w in words[1:] if not w.endswith(":")]
        try:
            return max(os.path.getmtime(f) for f in files) if files else 0.0
        except OSError:
            return float("inf")          # a header it used is gone: recompile
    hs = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return max(os.path.getmtime(h) for h in hs)


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
    if force or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), _deps_mtime(obj)):
        cmd = [HIPCC] + FLAGS + ["-MD", "-MF", obj + ".d", "-x", "hip", "-c", src, "-o", obj]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if out.strip():
            print(out)
    return obj


def build(jobs: int = 8, force: bool = False) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    srcs = sources()
    dsrcs = diag_sources()
    with cf.ThreadPoolExecutor(max_workers=max(1, min(jobs, 16))) as ex:
        allobjs = list(ex.map(lambda s: _compile(s, force), srcs + dsrcs))
    objs, dobjs = allobjs[:len(srcs)], allobjs[len(srcs):]
    for lib, obs in ((LIB, objs), (DIAG_LIB, dobjs)):
        if obs and (force or not os.path.exists(lib) or any(os.path.getmtime(o) > os.path.getmtime(lib) for o in obs)):
            subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib] + obs)
    return LIB


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("-j", type=int, default=8)
    ap.add_argument("--force", action="store_true")
    a = ap.parse_args()
    print(build(a.j, a.force))
