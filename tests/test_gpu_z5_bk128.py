"""GPU parity of the kernels with a k-tile of 128 (outside the default schedule space until they
have been measured): exact on integers for every such kernel, bit-identical across stage counts,
tolerance on the 2048^3 configuration."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV, ODT, TDT, assert_close, to_f64

pytestmark = pytest.mark.gpu


def _wide(prob):
    return [s for s in al.alcop_sched_variants(prob) if s.bk == 128 and al.alcop_sched_supported(prob, s) == al.OK]


@pytest.mark.parametrize("dt,transB", [("f16", False), ("bf16", False), ("f16", True), ("bf16", True)])
def test_integers_bit_exact_every_wide_kernel(dt, transB):
    it = al.F16 if dt == "f16" else al.BF16
    prob = al.problem(al.OP_GEMM, 512, 512, 1024, it, al.F32, transB=transB)
    scheds = _wide(prob)
    assert len(scheds) >= 1      # which rings fit the LDS depends on dtype and layout; every one is checked
    for n, s in enumerate(scheds):
        M, N, K = s.bm + 40, s.bn + 8, 3 * 128 + 8 if s.l2_prefetch == 0 else 5 * 128
        A = wl.small_ints((M, K), dt, 900 + n)
        B = wl.small_ints((N, K) if transB else (K, N), dt, 901 + n)
        ref = oracle.gemm(wl.bits(A), wl.bits(B.t().contiguous() if transB else B), ODT[dt])
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        al.alcop_gemm(A.to(DEV), B.to(DEV), C, s, transB=transB)
        torch.cuda.synchronize()
        assert np.array_equal(to_f64(C), ref), repr(s)


def test_random_bit_identical_across_pipelining_variants_and_close_on_gemm2048():
    cfg, A, B = wl.make_inputs("gemm2048")
    ref = oracle.gemm(wl.bits(A), wl.bits(B), ODT[cfg["dtype"]])
    Ad, Bd = A.to(DEV), B.to(DEV)
    prob = al.problem(al.OP_GEMM, 2048, 2048, 2048, al.F16, al.F16)
    by_tile = {}
    for s in _wide(prob):
        if s.l2_prefetch:
            continue
        C = torch.empty(2048, 2048, dtype=TDT[cfg["out"]], device=DEV)
        al.alcop_gemm(Ad, Bd, C, s)
        torch.cuda.synchronize()
        by_tile.setdefault((s.bm, s.bn, s.wm, s.wn), []).append((s, C))
    assert by_tile
    for tile, runs in by_tile.items():
        assert_close(to_f64(runs[0][1]), ref, "gemm2048 " + repr(runs[0][0]))
        for s, C in runs[1:]:          # same tile, same k order: stage count must not change a bit
            assert torch.equal(C.view(torch.int16), runs[0][1].view(torch.int16)), repr(s)
