"""The allocation-free split-K entry point (alcop_gemm_splitk_static) against alcop_gemm_splitk:
same kernels, the partial tiles in the library's own device array instead of a caller workspace.
Two calls in a row on one GPU, the second with a smaller problem, must each match the existing
entry point bit for bit (and that one is checked against the oracle); a problem whose partial
tiles exceed the array is refused on the host."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV, to_f64

pytestmark = pytest.mark.gpu


def _pair(M, N, K, split, seed, out=torch.float16, sched=None, ints=False, **epi):
    gen = wl.small_ints if ints else (lambda shape, dt, sd: wl.uniform(shape, dt, sd))
    A = gen((M, K), "f16", seed)
    B = gen((K, N), "f16", seed + 1)
    Ad, Bd = A.to(DEV), B.to(DEV)
    ws = torch.empty(al.alcop_splitk_workspace_bytes(1, M, N, max(split, 1) if split else 64) // 4,
                     dtype=torch.float32, device=DEV)
    want = torch.full((M, N), float("nan"), dtype=out, device=DEV)
    got = torch.full((M, N), float("nan"), dtype=out, device=DEV)
    al.alcop_gemm_splitk(Ad, Bd, want, split, ws, sched, **epi)
    al.alcop_gemm_splitk_static(Ad, Bd, got, split, sched, **epi)
    torch.cuda.synchronize()
    return A, B, want, got


def test_two_calls_in_a_row_match_the_workspace_entry_point_bit_for_bit():
    # first call: 1024 x 64 output, K = 2048, 16 slices (the small-output / long-K shape)
    A, B, want, got = _pair(1024, 64, 2048, 16, 4100)
    assert torch.equal(want.view(torch.int16), got.view(torch.int16))
    ref = oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16)
    assert np.all(np.abs(to_f64(got) - ref) <= 1e-2 * (np.abs(ref) + 1.0))
    # second call, smaller and ragged, other slice count, fp32 output, fused epilogue; what the
    # first call left in the array must not show
    bias = (torch.arange(72, dtype=torch.float32) - 30).to(DEV)
    A, B, want, got = _pair(136, 72, 7 * 64 + 8, 3, 4200, out=torch.float32, ints=True,
                            alpha=0.5, bias=bias, act=1)
    assert torch.equal(want.view(torch.int32), got.view(torch.int32))
    ref = oracle.epilogue(oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16), 0.5, bias.cpu().double().numpy(), 1)
    assert np.array_equal(to_f64(got), ref)
    # third: the first shape again (larger than the second), the model's choice of slices
    A, B, want, got = _pair(1024, 64, 2048, 0, 4300)
    assert torch.equal(want.view(torch.int16), got.view(torch.int16))


def test_batched_and_a_named_schedule():
    b, M, N, K = 3, 136, 72, 1000
    A = wl.small_ints((b, M, K), "f16", 4400)
    B = wl.small_ints((b, K, N), "f16", 4401)
    Ad, Bd = A.to(DEV), B.to(DEV)
    s = al.sched(128, 128, 64, 64, 64, 3, 2, 1)
    ws = torch.empty(al.alcop_splitk_workspace_bytes(b, M, N, 5) // 4, dtype=torch.float32, device=DEV)
    want = torch.full((b, M, N), float("nan"), dtype=torch.float32, device=DEV)
    got = torch.full((b, M, N), float("nan"), dtype=torch.float32, device=DEV)
    al.alcop_gemm_splitk(Ad, Bd, want, 5, ws, s)
    al.alcop_gemm_splitk_static(Ad, Bd, got, 5, s)
    torch.cuda.synchronize()
    assert torch.equal(want.view(torch.int32), got.view(torch.int32))
    ref = oracle.bmm(wl.bits(A), wl.bits(B), oracle.F16)
    assert np.array_equal(to_f64(got), ref)


def test_partial_tiles_beyond_the_array_are_refused():
    # 4 slices of 2048 x 2048 fp32 = 64 MiB > 32 MiB
    A = torch.zeros(2048, 256, dtype=torch.float16, device=DEV)
    B = torch.zeros(256, 2048, dtype=torch.float16, device=DEV)
    C = torch.zeros(2048, 2048, dtype=torch.float16, device=DEV)
    with pytest.raises(al.AlcopError) as e:
        al.alcop_gemm_splitk_static(A, B, C, 4)
    assert e.value.code == al.ERR_SIZE
    # two slices fit exactly (32 MiB)
    al.alcop_gemm_splitk_static(A, B, C, 2)
    torch.cuda.synchronize()
    assert torch.count_nonzero(C).item() == 0
