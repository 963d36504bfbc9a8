"""Shared helpers of the GPU parity tests (marshalling and comparison only)."""
import numpy as np
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl

DEV = "cuda:0"
ODT = {"f16": oracle.F16, "bf16": oracle.BF16}
ADT = {"f16": al.F16, "bf16": al.BF16, "f32": al.F32}
TDT = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}
RTOL = 1e-2   # |gpu - ref| <= 1e-2 * (|ref| + 1), the acceptance bound for random inputs


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


def assert_close(got: np.ndarray, ref: np.ndarray, what=""):
    assert got.shape == ref.shape
    assert np.all(np.isfinite(got)), what
    bound = RTOL * (np.abs(ref) + 1.0)
    bad = np.abs(got - ref) > bound
    assert not bad.any(), "%s: %d elements outside tolerance, worst %.3e" % (
        what, int(bad.sum()), float(np.max(np.abs(got - ref) / (np.abs(ref) + 1.0))))


def feasible(prob):
    return [s for s in al.alcop_sched_space(prob) if al.alcop_sched_supported(prob, s) == al.OK]


def tile_key(s):
    return (s.bm, s.bn, s.bk, s.wm, s.wn)
