"""GPU parity of the tiles 192 wide along n (three 64-column LDS images per stage): exact on
integers for every such kernel with ragged edges, and the transformer linear 4096 x 768 . 768 x 3072
at full size, where they give exactly one tile per compute unit, against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import ADT, DEV, ODT, TDT, assert_close, to_f64

pytestmark = pytest.mark.gpu


def _wide(prob):
    return [s for s in al.alcop_sched_space(prob) if s.bn == 192 and al.alcop_sched_supported(prob, s) == al.OK]


@pytest.mark.parametrize("dt,transB", [("f16", False), ("bf16", False), ("f16", True), ("bf16", True)])
def test_integers_bit_exact_every_wide_kernel(dt, transB):
    prob = al.problem(al.OP_GEMM, 1024, 768, 512, ADT[dt], al.F32, transB=transB)
    scheds = _wide(prob)
    assert scheds
    for n, s in enumerate(scheds):
        M, N, K = 2 * s.bm + 40, 3 * s.bn - (8, 72, 136)[n % 3], (1 + n % 5) * s.bk + (8 if n % 2 else 0)
        A = wl.small_ints((M, K), dt, 1900 + n)
        B = wl.small_ints((N, K) if transB else (K, N), dt, 1901 + n)
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        al.alcop_gemm(A.to(DEV), B.to(DEV), C, s, transB=transB)
        torch.cuda.synchronize()
        ref = oracle.gemm(wl.bits(A), wl.bits(B), ODT[dt], False, transB)
        assert np.array_equal(to_f64(C), ref), (repr(s), M, N, K)


def test_transformer_linear_full_size_one_tile_per_compute_unit():
    cfg, A, B = wl.make_inputs("ffn1")
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    assert (M // 256) * (N // 192) == 256
    ref = oracle.gemm(wl.bits(A), wl.bits(B), ODT[cfg["dtype"]])
    Ad, Bd = A.to(DEV), B.to(DEV)
    prob = al.problem(al.OP_GEMM, M, N, K, ADT[cfg["dtype"]], ADT[cfg["out"]])
    scheds = _wide(prob)
    first = None
    for s in scheds:
        C = torch.full((M, N), float("nan"), dtype=TDT[cfg["out"]], device=DEV)
        al.alcop_gemm(Ad, Bd, C, s)
        torch.cuda.synchronize()
        assert_close(to_f64(C), ref, repr(s))
        bits = C.view(torch.int16)
        if (s.bk, s.wm, s.wn) == (32, 128, 96):
            # one tile and k-tile: the same bits whatever the pipelining
            if first is None:
                first = bits.clone()
            else:
                assert torch.equal(bits, first), repr(s)
