"""GPU parity of alcop_bmm (attention-shaped batched matmuls) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV, TDT, assert_close, feasible, to_f64

pytestmark = pytest.mark.gpu


def run_bmm(A, B, out, s, transB):
    b, M = A.shape[0], A.shape[1]
    N = B.shape[1] if transB else B.shape[2]
    C = torch.full((b, M, N), float("nan"), dtype=TDT[out], device=DEV)
    al.alcop_bmm(A.to(DEV), B.to(DEV), C, s, transB=transB)
    torch.cuda.synchronize()
    return C


@pytest.mark.parametrize("transB", [True, False])
def test_integers_bit_exact_every_schedule(transB):
    b, M, N, K = 5, 192, 136, 128
    A = wl.small_ints((b, M, K), "f16", 201)
    B = wl.small_ints((b, N, K) if transB else (b, K, N), "f16", 202)
    ref = oracle.bmm(wl.bits(A), wl.bits(B), oracle.F16, transB=transB)
    prob = al.problem(al.OP_BMM, M, N, K, al.F16, al.F32, batch=b, transB=transB)
    for s in feasible(prob):
        assert np.array_equal(to_f64(run_bmm(A, B, "f32", s, transB)), ref), repr(s)


def test_config_bert_qk_full():
    cfg, Q, Km = wl.make_inputs("bmm_qk")
    ref = oracle.bmm(wl.bits(Q), wl.bits(Km), oracle.F16, transB=True)
    prob = al.problem(al.OP_BMM, 512, 512, 64, al.F16, al.F16, batch=96, transB=True)
    for s in [None] + feasible(prob)[::3]:
        got = to_f64(run_bmm(Q, Km, "f16", s, True))
        assert_close(got, ref, "bmm_qk " + repr(s))
    # the tolerance is loose for |values| ~ 0.1; also bound the error in units of the product scale
    got32 = to_f64(run_bmm(Q, Km, "f32", None, True))
    assert np.max(np.abs(got32 - ref)) < 2.0 ** -10 * np.sqrt(64) * 0.125 * 0.125


def test_config_bert_pv_full():
    cfg, P, V = wl.make_inputs("bmm_pv")
    ref = oracle.bmm(wl.bits(P), wl.bits(V), oracle.F16, transB=False)
    prob = al.problem(al.OP_BMM, 512, 64, 512, al.F16, al.F16, batch=96)
    for s in [None] + feasible(prob)[::3]:
        got = to_f64(run_bmm(P, V, "f16", s, False))
        assert_close(got, ref, "bmm_pv " + repr(s))
    got32 = to_f64(run_bmm(P, V, "f32", None, False))
    assert np.max(np.abs(got32 - ref)) < 1e-5


def test_qkt_symmetric_and_one_hot_gather():
    b, L, d = 4, 128, 64
    Q = wl.normal((b, L, d), "f16", 203, 0.125)
    S = run_bmm(Q, Q, "f32", al.sched(64, 64, 32, 32, 32, 2, 2, 1), True)
    assert torch.equal(S, S.transpose(1, 2))          # same products, same order: exact symmetry
    V = wl.normal((b, L, d), "f16", 204, 0.125)
    idx = torch.randint(0, L, (b, L), generator=torch.Generator().manual_seed(5))
    H = torch.zeros(b, L, L, dtype=torch.float16)
    H.scatter_(2, idx[:, :, None], 1.0)
    G = run_bmm(H, V, "f16", al.sched(64, 64, 32, 32, 32, 2, 2, 1), False)
    want = torch.gather(V, 1, idx[:, :, None].expand(b, L, d))
    assert torch.equal(G.cpu(), want)


def test_batch_strides_of_views():
    # batch entries taken from a larger buffer (stride larger than M*K)
    b, M, N, K = 3, 128, 128, 64
    big = wl.small_ints((b, M + 16, K), "f16", 205)
    A = big[:, :M, :]
    B = wl.small_ints((b, K, N), "f16", 206)
    ref = oracle.bmm(wl.bits(A.contiguous()), wl.bits(B), oracle.F16)
    C = torch.empty(b, M, N, dtype=torch.float32, device=DEV)
    al.alcop_bmm(big.to(DEV)[:, :M, :], B.to(DEV), C, al.sched(128, 128, 64, 64, 64, 1, 1, 0))
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(C), ref)
