"""GPU parity for A stored K x M (transA): the A tile is then M-contiguous in LDS and is read
with the transposing load, like a K x N B tile."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import ADT, DEV, ODT, TDT, assert_close, feasible, tile_key, to_f64

pytestmark = pytest.mark.gpu


def run(At, B, out, s, transB):
    M = At.shape[1]
    N = B.shape[0] if transB else B.shape[1]
    C = torch.full((M, N), float("nan"), dtype=TDT[out], device=DEV)
    al.alcop_gemm(At.to(DEV), B.to(DEV), C, s, transB=transB, transA=True)
    torch.cuda.synchronize()
    return C


@pytest.mark.parametrize("dt,transB", [("f16", False), ("f16", True), ("bf16", False), ("bf16", True)])
def test_integers_bit_exact_every_schedule(dt, transB):
    M, N, K = 256, 264, 200          # ragged N and a partial last k-tile
    At = wl.small_ints((K, M), dt, 601)
    B = wl.small_ints((N, K) if transB else (K, N), dt, 602)
    ref = oracle.gemm(wl.bits(At), wl.bits(B), ODT[dt], transA=True, transB=transB)
    prob = al.problem(al.OP_GEMM, M, N, K, ADT[dt], al.F32, transB=transB, transA=True)
    scheds = feasible(prob)
    assert len(scheds) >= 6
    for s in scheds:
        assert np.array_equal(to_f64(run(At, B, "f32", s, transB)), ref), repr(s)


def test_ragged_m_multiple_of_8():
    M, N, K = 200, 72, 128
    At = wl.small_ints((K, M), "f16", 603)
    B = wl.small_ints((K, N), "f16", 604)
    ref = oracle.gemm(wl.bits(At), wl.bits(B), oracle.F16, transA=True)
    for s in [al.sched(128, 128, 64, 64, 64, 3, 2, 1), al.sched(64, 64, 32, 32, 32, 2, 2, 1),
              al.sched(256, 256, 64, 128, 128, 2, 2, 1)]:
        assert np.array_equal(to_f64(run(At, B, "f32", s, False)), ref), repr(s)


def test_random_bit_identical_across_stages_and_equal_to_plain_layout():
    M, N, K = 512, 384, 640
    A = wl.uniform((M, K), "f16", 605)
    B = wl.uniform((K, N), "f16", 606)
    At = A.t().contiguous()
    ref = oracle.gemm(wl.bits(At), wl.bits(B), oracle.F16, transA=True)
    assert np.array_equal(ref, oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16))
    prob = al.problem(al.OP_GEMM, M, N, K, al.F16, al.F32, transA=True)
    groups = {}
    for s in feasible(prob):
        groups.setdefault(tile_key(s), []).append(s)
    for key, ss in groups.items():
        base = run(At, B, "f32", ss[0], False)
        assert_close(to_f64(base), ref, repr(ss[0]))
        for s in ss[1:]:
            assert torch.equal(base.view(torch.int32), run(At, B, "f32", s, False).view(torch.int32)), repr(s)
        # the same tile with A stored M x K performs the same products in the same order
        C0 = torch.empty(M, N, dtype=torch.float32, device=DEV)
        al.alcop_gemm(A.to(DEV), B.to(DEV), C0, ss[0])
        torch.cuda.synchronize()
        assert torch.equal(base.view(torch.int32), C0.view(torch.int32)), repr(ss[0])


def test_bmm_transa():
    b, M, N, K = 3, 128, 136, 96
    At = wl.small_ints((b, K, M), "f16", 607)
    B = wl.small_ints((b, K, N), "f16", 608)
    ref = oracle.bmm(wl.bits(At), wl.bits(B), oracle.F16, transA=True)
    C = torch.empty(b, M, N, dtype=torch.float32, device=DEV)
    al.alcop_bmm(At.to(DEV), B.to(DEV), C, al.sched(128, 128, 64, 64, 64, 3, 2, 1), transA=True)
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(C), ref)
