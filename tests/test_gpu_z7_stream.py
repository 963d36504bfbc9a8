"""GPU parity of the persistent producer / consumer kernels (schedule variant 2): exact on integers
for every such kernel and several numbers of persistent blocks, the same bits as the
tile-at-a-time kernel of the same tile on random data, and the attention / convolution
configurations at full size against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV, assert_close, to_f64

pytestmark = pytest.mark.gpu


def _stream(prob):
    # the default persistent kernels and the opt-in ones with the consumers' deep register pipeline
    both = al.alcop_sched_space(prob) + al.alcop_sched_variants(prob)
    return [s for s in both if s.variant == 2 and al.alcop_sched_supported(prob, s) == al.OK]


@pytest.mark.parametrize("dt,transB", [("f16", False), ("f16", True), ("bf16", False)])
def test_integers_bit_exact_every_stream_kernel_and_block_count(dt, transB, monkeypatch):
    it = al.F16 if dt == "f16" else al.BF16
    prob = al.problem(al.OP_BMM, 512, 512, 512, it, al.F32, batch=5, transB=transB)
    scheds = _stream(prob)
    assert scheds
    odt = oracle.F16 if dt == "f16" else oracle.BF16
    for n, s in enumerate(scheds):
        b, M, N, K = 5, 3 * s.bm + 24, 2 * s.bn + 8, (1 + n % 4) * s.bk + (8 if n % 2 else 0)
        A = wl.small_ints((b, M, K), dt, 1400 + n)
        B = wl.small_ints((b, N, K) if transB else (b, K, N), dt, 1401 + n)
        ref = oracle.bmm(wl.bits(A), wl.bits(B), odt, transB=transB)
        Ad, Bd = A.to(DEV), B.to(DEV)
        for blocks in ("1", "7", "64", None):
            if blocks is None:
                monkeypatch.delenv("ALCOP_STREAM_BLOCKS", raising=False)
            else:
                monkeypatch.setenv("ALCOP_STREAM_BLOCKS", blocks)
            C = torch.full((b, M, N), float("nan"), dtype=torch.float32, device=DEV)
            al.alcop_bmm(Ad, Bd, C, s, transB=transB)
            torch.cuda.synchronize()
            assert np.array_equal(to_f64(C), ref), (repr(s), blocks, K)


def test_convolution_integers_bit_exact_every_stream_kernel(monkeypatch):
    N, H, W, C, K = 3, 17, 15, 64, 72
    x = wl.small_ints((N, H, W, C), "f16", 1410)
    w = wl.small_ints((3, 3, C, K), "f16", 1411)
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (1, 1), (1, 1))
    prob = al.problem(al.OP_CONV2D, N * H * W, K, 9 * C, al.F16, al.F32, conv_C=C)
    scheds = _stream(prob)
    assert scheds
    xd, wd = x.to(DEV), w.to(DEV)
    for s in scheds:
        for blocks in ("3", None):
            if blocks is None:
                monkeypatch.delenv("ALCOP_STREAM_BLOCKS", raising=False)
            else:
                monkeypatch.setenv("ALCOP_STREAM_BLOCKS", blocks)
            y = torch.full((N, H, W, K), float("nan"), dtype=torch.float32, device=DEV)
            al.alcop_conv2d_igemm(xd, wd, y, (1, 1), (1, 1), s)
            torch.cuda.synchronize()
            assert np.array_equal(to_f64(y), ref), (repr(s), blocks)


def test_same_bits_as_the_tile_at_a_time_kernel_on_random_data():
    b, M, N, K = 7, 392, 264, 328
    A = wl.normal((b, M, K), "f16", 1420, 0.5)
    B = wl.normal((b, K, N), "f16", 1421, 0.5)
    ref = oracle.bmm(wl.bits(A), wl.bits(B), oracle.F16)
    prob = al.problem(al.OP_BMM, M, N, K, al.F16, al.F16, batch=b)
    Ad, Bd = A.to(DEV), B.to(DEV)
    for s in _stream(prob):
        C = torch.full((b, M, N), float("nan"), dtype=torch.float16, device=DEV)
        al.alcop_bmm(Ad, Bd, C, s)
        plain = al.sched(s.bm, s.bn, s.bk, s.wm, s.wn, 2, 2, 1)
        if al.alcop_sched_supported(prob, plain) != al.OK:
            plain = al.sched(s.bm, s.bn, s.bk, s.wm, s.wn, 1, 1, 0)
        D = torch.full((b, M, N), float("nan"), dtype=torch.float16, device=DEV)
        al.alcop_bmm(Ad, Bd, D, plain)
        torch.cuda.synchronize()
        assert torch.equal(C.view(torch.int16), D.view(torch.int16)), repr(s)
        assert_close(to_f64(C), ref, repr(s))


@pytest.mark.parametrize("name", ["bmm_qk", "bmm_pv", "conv56", "conv14"])
def test_configurations_full_size(name):
    cfg, A, B = wl.make_inputs(name)
    Ad, Bd = A.to(DEV), B.to(DEV)
    if cfg["kind"] == "bmm":
        ref = oracle.bmm(wl.bits(A), wl.bits(B), oracle.F16, transB=cfg["transB"])
        prob = al.problem(al.OP_BMM, cfg["M"], cfg["N"], cfg["K"], al.F16, al.F16, batch=cfg["batch"],
                          transB=cfg["transB"])
    else:
        ref = oracle.conv2d(wl.bits(A), wl.bits(B), oracle.F16, (1, 1), (1, 1))
        n, H, W, C, Ko = (cfg[k] for k in ("N", "H", "W", "C", "K"))
        prob = al.problem(al.OP_CONV2D, n * H * W, Ko, 9 * C, al.F16, al.F16, conv_C=C)
    scheds = _stream(prob)
    assert scheds
    for s in scheds[::3]:
        out = torch.full(tuple(ref.shape), float("nan"), dtype=torch.float16, device=DEV)
        if cfg["kind"] == "bmm":
            al.alcop_bmm(Ad, Bd, out, s, transB=cfg["transB"])
        else:
            al.alcop_conv2d_igemm(Ad, Bd, out, (1, 1), (1, 1), s)
        torch.cuda.synchronize()
        assert_close(to_f64(out), ref, name + " " + repr(s))
