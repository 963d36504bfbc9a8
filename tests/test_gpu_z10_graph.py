"""The entry points allocate nothing and never synchronise, so a caller may record them into a HIP
graph.  A GEMM, the allocation-free split-K product and a persistent batched product are captured
once and replayed several times on changing inputs, with eager work and synchronisation between
the replays; every replay must equal the eager result bit for bit."""
import pytest
import torch

import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV

pytestmark = pytest.mark.gpu


def test_captured_launches_replay_bit_identically():
    M, N, K, b = 384, 264, 520, 3
    A = wl.uniform((M, K), "f16", 9201).to(DEV)
    B = wl.uniform((K, N), "f16", 9202).to(DEV)
    Ab = wl.uniform((b, M, K), "f16", 9203).to(DEV)
    Bb = wl.uniform((b, K, N), "f16", 9204).to(DEV)
    C1 = torch.empty(M, N, dtype=torch.float16, device=DEV)
    C2 = torch.empty(M, N, dtype=torch.float16, device=DEV)
    C3 = torch.empty(b, M, N, dtype=torch.float16, device=DEV)
    s_plain = al.sched(128, 128, 64, 64, 64, 3, 2, 1)
    s_stream = al.sched(128, 128, 64, 64, 64, 3, 2, 1, 1, 0, 2)

    def work(stream):
        al.alcop_gemm(A, B, C1, s_plain, stream=stream)
        al.alcop_gemm_splitk_static(A, B, C2, 3, stream=stream)
        al.alcop_bmm(Ab, Bb, C3, s_stream, stream=stream)

    work(torch.cuda.current_stream())          # first launches opt the kernels in to their LDS size
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        work(side)                              # warm on the capture stream too
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            work(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(4):
        # new operand values in place, eager reference, then the replay
        A.copy_(wl.uniform((M, K), "f16", 9300 + rep).to(DEV))
        Bb.copy_(wl.uniform((b, K, N), "f16", 9400 + rep).to(DEV))
        work(torch.cuda.current_stream())
        torch.cuda.synchronize()
        want = [C1.clone(), C2.clone(), C3.clone()]
        for t in (C1, C2, C3):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref, what in zip((C1, C2, C3), want, ("gemm", "split-K static", "persistent bmm")):
            assert torch.equal(got.view(torch.int16), ref.view(torch.int16)), (what, rep)


def test_capture_without_an_eager_call_after_alcop_init():
    al.alcop_init()
    M, N, K = 512, 384, 256
    A = wl.uniform((M, K), "bf16", 9501).to(DEV)
    B = wl.uniform((K, N), "bf16", 9502).to(DEV)
    C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    s = al.sched(256, 192, 64, 64, 96, 2, 2, 1)      # a kernel no other call of this file launches
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            al.alcop_gemm(A, B, C, s, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(3):
        graph.replay()
        torch.cuda.synchronize()
        got = C.clone()
        C.fill_(float("nan"))
        al.alcop_gemm(A, B, C, s)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), C.view(torch.int16)), rep
        A.copy_(wl.uniform((M, K), "bf16", 9600 + rep).to(DEV))
        C.fill_(float("nan"))
