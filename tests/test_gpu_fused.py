"""GPU parity of the consumer-side fused elementwise epilogue (scale, bias, ReLU)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV, assert_close, to_f64

pytestmark = pytest.mark.gpu

SCHEDS = [al.sched(128, 128, 64, 64, 64, 3, 2, 1), al.sched(64, 64, 32, 32, 32, 1, 1, 0),
          al.sched(256, 256, 32, 128, 64, 4, 2, 1), None]


def test_integers_exact_scale_bias_relu():
    M, N, K = 200, 136, 128
    A = wl.small_ints((M, K), "f16", 501)
    B = wl.small_ints((K, N), "f16", 502)
    bias = torch.randint(-40, 41, (N,), generator=torch.Generator().manual_seed(503)).float()
    base = oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16)
    for alpha, use_bias, act in [(0.5, True, 1), (2.0, False, 0), (1.0, True, 0), (1.0, False, 1), (-1.0, True, 1)]:
        ref = oracle.epilogue(base, alpha, bias.numpy() if use_bias else None, act)
        for s in SCHEDS:
            C = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
            al.alcop_gemm_fused(A.to(DEV), B.to(DEV), C, alpha, bias.to(DEV) if use_bias else None, act, s)
            torch.cuda.synchronize()
            assert np.array_equal(to_f64(C), ref), (alpha, use_bias, act, repr(s))


def test_default_epilogue_equals_plain_gemm():
    A = wl.uniform((256, 256), "f16", 504)
    B = wl.uniform((256, 256), "f16", 505)
    s = al.sched(128, 128, 64, 64, 64, 3, 2, 1)
    C0 = torch.empty(256, 256, dtype=torch.float16, device=DEV)
    C1 = torch.empty_like(C0)
    al.alcop_gemm(A.to(DEV), B.to(DEV), C0, s)
    al.alcop_gemm_fused(A.to(DEV), B.to(DEV), C1, 1.0, None, 0, s)
    torch.cuda.synchronize()
    assert torch.equal(C0.view(torch.int16), C1.view(torch.int16))


def test_attention_scores_scaled():
    # Q.K^T / sqrt(d) with the scale fused (BERT-base head: d = 64)
    cfg, Q, Km = wl.make_inputs("bmm_qk", batch=8)
    ref = oracle.epilogue(oracle.bmm(wl.bits(Q), wl.bits(Km), oracle.F16, transB=True), 0.125)
    C = torch.empty(8, 512, 512, dtype=torch.float16, device=DEV)
    al.alcop_bmm_fused(Q.to(DEV), Km.to(DEV), C, 0.125, None, 0, None, transB=True)
    torch.cuda.synchronize()
    assert_close(to_f64(C), ref, "scaled scores")
    assert np.max(np.abs(to_f64(C) - ref)) < 2e-3


def test_linear_layer_bias_relu_bf16():
    A = wl.uniform((512, 768), "bf16", 506)
    W = wl.uniform((768, 1024), "bf16", 507)
    bias = torch.randn(1024, generator=torch.Generator().manual_seed(508))
    ref = oracle.epilogue(oracle.gemm(wl.bits(A), wl.bits(W), oracle.BF16), 1.0, bias.numpy(), 1)
    C = torch.empty(512, 1024, dtype=torch.bfloat16, device=DEV)
    al.alcop_gemm_fused(A.to(DEV), W.to(DEV), C, 1.0, bias.to(DEV), 1, None)
    torch.cuda.synchronize()
    got = to_f64(C)
    assert_close(got, ref, "bias+relu")
    assert (got >= 0).all() and (got == 0).any()
