"""GPU parity of the split-K entry points (alcop_gemm_splitk, alcop_conv2d_igemm_splitk) against
the oracle: exact on integer inputs for every variant and several slice counts, tolerance on the
paper's small-output / long-reduction shape and on the small-output convolution."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV, ODT, TDT, assert_close, to_f64

pytestmark = pytest.mark.gpu


def _ws(batch, M, N, split):
    n = al.alcop_splitk_workspace_bytes(batch, M, N, split)
    return torch.full((n // 4,), float("nan"), dtype=torch.float32, device=DEV)


@pytest.mark.parametrize("dt,transB", [("f16", False), ("f16", True), ("bf16", False), ("bf16", True)])
def test_integers_bit_exact_every_variant(dt, transB):
    prob = al.problem(al.OP_GEMM, 512, 512, 1024, al.F16 if dt == "f16" else al.BF16, al.F32, transB=transB)
    scheds = al.alcop_splitk_space(prob)
    assert scheds
    for n, s in enumerate(scheds):
        M, N, K = s.bm + 24, s.bn + 8, 9 * 64 + 24
        A = wl.small_ints((M, K), dt, 700 + n)
        B = wl.small_ints((N, K) if transB else (K, N), dt, 701 + n)
        ref = oracle.gemm(wl.bits(A), wl.bits(B.t().contiguous() if transB else B), ODT[dt])
        Ad, Bd = A.to(DEV), B.to(DEV)
        for split in (2, 5, 10):
            C = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
            al.alcop_gemm_splitk(Ad, Bd, C, split, _ws(1, M, N, split), s, transB=transB)
            torch.cuda.synchronize()
            assert np.array_equal(to_f64(C), ref), (repr(s), split)


def test_split_one_equals_unsplit_kernel_bitwise_and_runs_are_deterministic():
    M, N, K = 256, 192, 1024
    A = wl.uniform((M, K), "f16", 711).to(DEV)
    B = wl.uniform((K, N), "f16", 712).to(DEV)
    s = al.sched(128, 128, 64, 64, 64, 3, 2, 1)
    ref = torch.empty(M, N, dtype=torch.float16, device=DEV)
    al.alcop_gemm(A, B, ref, s)
    C1 = torch.empty_like(ref)
    al.alcop_gemm_splitk(A, B, C1, 1, _ws(1, M, N, 1), s)
    torch.cuda.synchronize()
    assert torch.equal(C1.view(torch.int16), ref.view(torch.int16))     # one slice: same k order
    runs = []
    for _ in range(5):
        C = torch.empty_like(ref)
        al.alcop_gemm_splitk(A, B, C, 4, _ws(1, M, N, 4), s)
        torch.cuda.synchronize()
        runs.append(C.view(torch.int16).clone())
    assert all(torch.equal(r, runs[0]) for r in runs[1:])


def test_paper_best_case_shape_small_output_long_k():
    # 1024 x 64 output, K = 2048 (paper Sec. 6.2): 16 tiles of 64 x 64 without slicing
    cfg, A, B = wl.make_inputs("mm_rn50_fc")
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    ref = oracle.gemm(wl.bits(A), wl.bits(B), ODT[cfg["dtype"]])
    Ad, Bd = A.to(DEV), B.to(DEV)
    prob = al.problem(al.OP_GEMM, M, N, K, al.F16, al.F16)
    s, split, us = al.alcop_splitk_auto(prob)
    assert split > 1
    C = torch.full((M, N), float("nan"), dtype=TDT[cfg["out"]], device=DEV)
    al.alcop_gemm_splitk(Ad, Bd, C, split, _ws(1, M, N, split), s)
    torch.cuda.synchronize()
    assert_close(to_f64(C), ref, "mm_rn50_fc split %d %r" % (split, s))
    # schedule and split both left to the library
    C2 = torch.full((M, N), float("nan"), dtype=TDT[cfg["out"]], device=DEV)
    al.alcop_gemm_splitk(Ad, Bd, C2, 0, _ws(1, M, N, 64), None)
    torch.cuda.synchronize()
    assert_close(to_f64(C2), ref, "mm_rn50_fc auto")


def test_fused_epilogue_and_batched():
    b, M, N, K = 3, 72, 136, 5 * 64
    A = wl.small_ints((b, M, K), "bf16", 721)
    B = wl.small_ints((b, K, N), "bf16", 722)
    bias = (torch.arange(N, dtype=torch.float32) % 7) - 3
    ref = oracle.epilogue(oracle.bmm(wl.bits(A), wl.bits(B), oracle.BF16), 0.25, bias.double().numpy(), 1)
    C = torch.full((b, M, N), float("nan"), dtype=torch.float32, device=DEV)
    al.alcop_gemm_splitk(A.to(DEV), B.to(DEV), C, 3, _ws(b, M, N, 3), al.sched(128, 128, 64, 64, 64, 2, 2, 1),
                         0.25, bias.to(DEV), 1)
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(C), ref)


def test_conv_integers_exact_and_config_conv14():
    g = dict(N=1, H=7, W=9, C=128, K=72, R=3, S=3, stride=(1, 1), pad=(1, 1))
    x = wl.small_ints((g["N"], g["H"], g["W"], g["C"]), "f16", 731)
    w = wl.small_ints((g["R"], g["S"], g["C"], g["K"]), "f16", 732)
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, g["stride"], g["pad"])
    M = g["N"] * g["H"] * g["W"]
    prob = al.problem(al.OP_CONV2D, M, g["K"], 9 * g["C"], al.F16, al.F32, conv_C=g["C"])
    xd, wd = x.to(DEV), w.to(DEV)
    for s in al.alcop_splitk_space(prob):
        for split in (2, 3, 18):
            y = torch.full((g["N"], g["H"], g["W"], g["K"]), float("nan"), dtype=torch.float32, device=DEV)
            al.alcop_conv2d_igemm_splitk(xd, wd, y, split, _ws(1, M, g["K"], split), g["stride"], g["pad"], s)
            torch.cuda.synchronize()
            assert np.array_equal(to_f64(y), ref), (repr(s), split)
    # the 14 x 14 x 256 layer of the configurations: 98 tiles of 128 x 128 without slicing
    cfg, x, w = wl.make_inputs("conv14")
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), ODT[cfg["dtype"]], (1, 1), (1, 1))
    n, H, W, K = cfg["N"], cfg["H"], cfg["W"], cfg["K"]
    y = torch.full((n, H, W, K), float("nan"), dtype=TDT[cfg["out"]], device=DEV)
    al.alcop_conv2d_igemm_splitk(x.to(DEV), w.to(DEV), y, 4, _ws(1, n * H * W, K, 4), (1, 1), (1, 1), None)
    torch.cuda.synchronize()
    assert_close(to_f64(y), ref, "conv14 split 4")
    scale = float(np.sqrt(np.mean(ref ** 2)))
    assert np.max(np.abs(to_f64(y) - ref)) < 2e-2 * scale


def test_bad_arguments_are_refused():
    A = torch.zeros(128, 256, dtype=torch.float16, device=DEV)
    B = torch.zeros(256, 64, dtype=torch.float16, device=DEV)
    C = torch.zeros(128, 64, dtype=torch.float16, device=DEV)
    small = torch.zeros(100, dtype=torch.float32, device=DEV)
    with pytest.raises(al.AlcopError) as e:
        al.alcop_gemm_splitk(A, B, C, 2, small, None)
    assert e.value.code == al.ERR_SIZE
    with pytest.raises(al.AlcopError) as e:
        al.alcop_gemm_splitk(A, B, C, 65, _ws(1, 128, 64, 4), None)
    assert e.value.code == al.ERR_SHAPE
    with pytest.raises(al.AlcopError) as e:      # not a split-K variant
        al.alcop_gemm_splitk(A, B, C, 2, _ws(1, 128, 64, 2), al.sched(256, 256, 32, 128, 64, 2, 2, 1))
    assert e.value.code == al.ERR_SCHED


def test_tuner_over_variants_and_slices():
    cfg, A, B = wl.make_inputs("mm_rn50_fc")
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    Ad, Bd = A.to(DEV), B.to(DEV)
    C = torch.empty(M, N, dtype=torch.float16, device=DEV)
    prob = al.problem(al.OP_GEMM, M, N, K, al.F16, al.F16)
    ws = _ws(1, M, N, 32)
    r, split = al.alcop_tune_splitk(prob, Ad, Bd, C, ws, top_k=8, iters=20)
    assert r.trials == 8 and len(r.log) == 8 and r.space > 8
    preds = [p for _, _, p, _ in r.log]
    assert preds == sorted(preds)                      # trials come in the model's order
    assert r.best_us == min(m for _, _, _, m in r.log)
    assert (r.best.key(), split) in [(s.key(), k) for s, k, _, _ in r.log]
    # a small workspace prunes the large slice counts
    tiny = _ws(1, M, N, 2)
    r2, split2 = al.alcop_tune_splitk(prob, Ad, Bd, C, tiny, top_k=0, iters=5)
    assert split2 <= 2 and all(k <= 2 for _, k, _, _ in r2.log) and r2.space < r.space
    # the tuned pair computes the right thing
    al.alcop_gemm_splitk(Ad, Bd, C, split, ws, r.best)
    torch.cuda.synchronize()
    assert_close(to_f64(C), oracle.gemm(wl.bits(A), wl.bits(B), ODT[cfg["dtype"]]), "tuned split-K")


def test_weight_gradient_layout_a_stored_k_by_m():
    # dW = X^T . dY with X [tokens, in] and dY [tokens, out]: A stored K x M, B stored K x N
    tokens, fin, fout = 8 * 64 + 40, 136, 72
    for dt in ("f16", "bf16"):
        X = wl.small_ints((tokens, fin), dt, 741)
        dY = wl.small_ints((tokens, fout), dt, 742)
        ref = oracle.gemm(wl.bits(X.t().contiguous()), wl.bits(dY), ODT[dt])
        prob = al.problem(al.OP_GEMM, fin, fout, tokens, al.F16 if dt == "f16" else al.BF16, al.F32, transA=True)
        scheds = al.alcop_splitk_space(prob)
        assert len(scheds) >= 6
        Xd, Yd = X.to(DEV), dY.to(DEV)
        for s in scheds:
            for split in (3, 9):
                dW = torch.full((fin, fout), float("nan"), dtype=torch.float32, device=DEV)
                al.alcop_gemm_splitk(Xd, Yd, dW, split, _ws(1, fin, fout, split), s, transA=True)
                torch.cuda.synchronize()
                assert np.array_equal(to_f64(dW), ref), (dt, repr(s), split)
