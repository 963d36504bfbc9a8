"""The static performance model (paper Sec. 5, Table 1): oracle pins by hand-computed values,
then the library's C++ model against the oracle over the whole schedule space (host only)."""
import math

import pytest

import paper_2210_16691_amd as al
from oracle import perf_model as pm


# ---- pins of the oracle ------------------------------------------------------------------------
def test_pipeline_latency_hand_values():
    # (3*1-1)*5 = 10 >= 10 -> compute bound: 5*8
    assert pm.pipeline_latency(10, 5, 8, 3, 1) == 40
    # 11 > 10 -> load bound: (11+5)*8/3
    assert pm.pipeline_latency(11, 5, 8, 3, 1) == pytest.approx(16 * 8 / 3)
    # multiplexing counts like extra stages: (2*2-1)*5 = 15 >= 11
    assert pm.pipeline_latency(11, 5, 8, 2, 2) == 40
    # one stage, one worker: nothing overlaps, load + use every iteration
    assert pm.pipeline_latency(7, 3, 10, 1, 1) == 100
    # zero load time is always hidden
    assert pm.pipeline_latency(0, 3, 10, 1, 1) == 30


def test_two_printed_forms_of_the_criterion_agree():
    for tl in [0, 1, 4.9, 5, 5.1, 9.99, 10, 10.01, 50]:
        for tu in [0.5, 1, 5]:
            for npipe in [1, 2, 3, 4]:
                for nm in [1, 2, 4]:
                    a = pm.pipeline_latency(tl, tu, 7, npipe, nm)
                    b = pm.pipeline_latency_caption_form(tl, tu, 7, npipe, nm)
                    assert a == b


def test_table_rows_by_hand():
    # 2048^3 fp16 -> fp16, 128x128x64 tile, 64x64 waves, S=3, R=2, fused; constants of pm.Device
    d = pm.Device()
    r = pm.predict(2048, 2048, 2048, 1, 2, 128, 128, 64, 64, 64, 3, 2, True, d)
    # scheduler: 256 blocks on 256 CUs -> one block per CU, one batch
    assert r["n_blk_per_cu"] == 1 and r["n_threadblk_batch"] == 1
    # compute: 2*128*128*16 flop on 4096 flop/clk * 1800 clk/us, 4 waves fill the 4 pipes
    assert r["util"] == 1.0
    assert r["t_compute"] == pytest.approx(524288 / (4096 * 1800.0))
    # register load: 128 clk latency + 4 waves * (64+64)*16*2 B at 128 B/clk
    assert r["t_reg_load"] == pytest.approx((128 + 16384 / 128) / 1800.0)
    # inner pipeline, R=2, one wave per pipe: hidden iff t_reg_load <= t_compute
    assert r["t_reg_load"] > r["t_compute"]
    t_pipe = (r["t_reg_load"] + r["t_compute"]) * 4 / 2
    # LDS port: A 128x64x2 B read by 2 waves along n at 128 B/clk, B likewise at 240 B/clk,
    # plus the 32 KiB k-tile written at 128 B/clk
    t_port = (32768 / 128 + 32768 / 240 + 32768 / 128) / 1800.0
    assert r["t_smem_use"] == pytest.approx(max(t_pipe, t_port))
    # memory: LLC term 0.6 + 256 blocks * 32 KiB / 16e6 ; DRAM term 1.2 + (16+16 panels)*128*64*2/8e6
    t_llc = 0.6 + 256 * 32768 / 16.0e6
    t_dram = 1.2 + 32 * 128 * 64 * 2 / 8.0e6
    assert r["t_smem_load"] == pytest.approx(max(t_llc, t_dram))
    assert r["t_init"] == pytest.approx(r["t_smem_load"] + r["t_reg_load"])
    # outer pipeline: 32 iterations, 3 stages, no multiplexing
    assert r["t_main_loop"] == pytest.approx(
        pm.pipeline_latency(r["t_smem_load"], r["t_smem_use"], 32, 3, 1))
    # epilogue: 1.0 + 256 tiles * 128*128*2 B / 8e6
    assert r["t_epilogue"] == pytest.approx(1.0 + 256 * 32768 / 8.0e6)
    assert r["t_kernel"] == pytest.approx(r["t_init"] + r["t_main_loop"] + r["t_epilogue"])


def test_model_monotone_in_stages_when_load_bound():
    # same tile, more stages never predicted slower as long as occupancy is unchanged
    prev = None
    for S in [1, 2, 3, 4]:
        t = pm.predict(2048, 2048, 2048, 1, 2, 128, 128, 32, 64, 64, S, 2, S >= 2)["t_kernel"]
        if prev is not None:
            assert t <= prev + 1e-12
        prev = t


def test_compute_bound_branch_ignores_load_time():
    a = pm.pipeline_latency(1.0, 10.0, 16, 2, 1)
    b = pm.pipeline_latency(9.0, 10.0, 16, 2, 1)
    assert a == b == 160.0


# ---- the library's model against the oracle ------------------------------------------------------
PROBLEMS = [
    dict(op=al.OP_GEMM, M=2048, N=2048, K=2048, i=al.F16, o=al.F16, batch=1, tb=False),
    dict(op=al.OP_GEMM, M=8192, N=8192, K=8192, i=al.BF16, o=al.BF16, batch=1, tb=False),
    dict(op=al.OP_GEMM, M=4096, N=768, K=3072, i=al.BF16, o=al.BF16, batch=1, tb=False),
    dict(op=al.OP_GEMM, M=1000, N=264, K=512, i=al.F16, o=al.F32, batch=1, tb=False),
    dict(op=al.OP_BMM, M=512, N=512, K=64, i=al.F16, o=al.F16, batch=96, tb=True),
    dict(op=al.OP_BMM, M=512, N=64, K=512, i=al.F16, o=al.F16, batch=96, tb=False),
    dict(op=al.OP_GEMM, M=2048, N=2048, K=2048, i=al.F16, o=al.F16, batch=1, tb=False, ta=True),
    dict(op=al.OP_GEMM, M=1024, N=512, K=4096, i=al.BF16, o=al.F32, batch=1, tb=True, ta=True),
]


@pytest.mark.parametrize("P", PROBLEMS)
def test_library_model_matches_oracle(P):
    prob = al.problem(P["op"], P["M"], P["N"], P["K"], P["i"], P["o"], batch=P["batch"], transB=P["tb"],
                      transA=P.get("ta", False))
    space = al.alcop_sched_space(prob)
    assert len(space) > 0
    ob = 4 if P["o"] == al.F32 else 2
    for s in space:
        us, terms = al.alcop_model_predict(prob, s, 0)
        r = pm.predict(P["M"], P["N"], P["K"], P["batch"], ob, s.bm, s.bn, s.bk, s.wm, s.wn,
                       s.stages, s.reg_stages, bool(s.fuse_inner), transB=P["tb"],
                       transA=P.get("ta", False))
        want = [r[k] for k in ("t_kernel", "t_threadblk", "t_init", "t_main_loop", "t_epilogue",
                               "t_smem_load", "t_smem_use", "n_threadblk_batch")]
        assert us == pytest.approx(r["t_kernel"], rel=1e-12)
        for g, w in zip(terms, want):
            assert g == pytest.approx(w, rel=1e-12)
        us1, _ = al.alcop_model_predict(prob, s, 1)
        assert us1 == pytest.approx(
            pm.bottleneck(P["M"], P["N"], P["K"], P["batch"], ob, s.bm, s.bn, s.bk, s.wm, s.wn), rel=1e-12)


@pytest.mark.parametrize("shape", [(1, 1024, 64, 2048), (1, 4096, 768, 3072), (3, 136, 72, 1000), (1, 2048, 2048, 2048)])
def test_library_splitk_model_matches_oracle(shape):
    b, M, N, K = shape
    prob = al.problem(al.OP_BMM if b > 1 else al.OP_GEMM, M, N, K, al.F16, al.F16, batch=b)
    for split in (1, 2, 5, 16, 64):
        s, k, us = al.alcop_splitk_auto(prob, split)
        assert k == split
        want, slices = pm.predict_splitk(M, N, K, b, 2, s.bm, s.bn, s.bk, s.wm, s.wn, s.stages,
                                         s.reg_stages, bool(s.fuse_inner), split)
        assert us == pytest.approx(want, rel=1e-12)
        # the pick is the arg-min of the same formula over the variants built for this problem
        best = min(pm.predict_splitk(M, N, K, b, 2, v.bm, v.bn, v.bk, v.wm, v.wn, v.stages, v.reg_stages,
                                     bool(v.fuse_inner), split)[0] for v in al.alcop_splitk_space(prob))
        assert us == pytest.approx(best, rel=1e-12)
    # hand-checked slicing: 33 k-tiles of 64 over 4 requested slices -> 9 per slice -> 4 slices;
    # over 16 requested -> 3 per slice -> 11 slices
    assert pm.predict_splitk(128, 128, 33 * 64, 1, 2, 128, 128, 64, 64, 64, 3, 2, True, 4)[1] == 4
    assert pm.predict_splitk(128, 128, 33 * 64, 1, 2, 128, 128, 64, 64, 64, 3, 2, True, 16)[1] == 11


def test_library_patch_convolution_model_matches_oracle():
    # conv 56x56x64 -> 64, 3x3: 9 taps; variant 1 fetches the A rows once per block
    M, N, K, C = 32 * 56 * 56, 64, 576, 64
    prob = al.problem(al.OP_CONV2D, M, N, K, al.F16, al.F16, conv_C=C)
    seen = 0
    for s in al.alcop_sched_space(prob) + al.alcop_sched_variants(prob):
        us, terms = al.alcop_model_predict(prob, s, 0)
        r = pm.predict(M, N, K, 1, 2, s.bm, s.bn, s.bk, s.wm, s.wn, s.stages, s.reg_stages,
                       bool(s.fuse_inner), patch_taps=9 if s.variant == 1 else 0)
        assert us == pytest.approx(r["t_kernel"], rel=1e-12)
        if s.variant == 1:
            seen += 1
            # less traffic per k-tile than the default kernel of the same schedule
            plain = al.sched(s.bm, s.bn, s.bk, s.wm, s.wn, s.stages, s.reg_stages, s.fuse_inner)
            assert terms[5] < al.alcop_model_predict(prob, plain, 0)[1][5]
    assert seen >= 6
