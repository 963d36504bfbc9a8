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
    # register load: 128 clk latency + 4 waves * (64+64)*16*2 B at 256 B/clk
    assert r["t_reg_load"] == pytest.approx((128 + 16384 / 256) / 1800.0)
    # inner pipeline, R=2, one wave per pipe: hidden iff t_reg_load <= t_compute
    assert r["t_reg_load"] > r["t_compute"]
    t_pipe = (r["t_reg_load"] + r["t_compute"]) * 4 / 2
    # LDS port: A 128x64x2 B read by 2 waves along n at 256 B/clk, B likewise at 170 B/clk
    # (transposing read), plus the 32 KiB k-tile written at 256 B/clk
    t_port = (32768 / 256 + 32768 / 170 + 32768 / 256) / 1800.0
    # fill path of the compute unit: the 32 KiB k-tile at 40 B/clk
    t_fill = 32768 / 40 / 1800.0
    assert t_fill > t_port and t_fill > t_pipe
    assert r["t_smem_use"] == pytest.approx(max(t_pipe, t_port, t_fill))
    # memory: LLC term 0.6 + 256 blocks * 32 KiB at 40 B/clk per CU ; DRAM term 1.2 + (16+16 panels)*128*64*2/8e6
    t_llc = 0.6 + 256 * 32768 / (40 * 256 * 1800.0)
    t_dram = 1.2 + 32 * 128 * 64 * 2 / 8.0e6
    assert r["t_smem_load"] == pytest.approx(max(t_llc, t_dram))
    assert r["t_init"] == pytest.approx(r["t_smem_load"] + r["t_reg_load"])
    # outer pipeline: 32 iterations, 3 stages, no multiplexing
    assert r["t_main_loop"] == pytest.approx(
        pm.pipeline_latency(r["t_smem_load"], r["t_smem_use"], 32, 3, 1))
    # epilogue: 1.0 + 256 tiles * 128*128*2 B / 8e6
    assert r["t_epilogue"] == pytest.approx(1.0 + 256 * 32768 / 8.0e6)
    assert r["t_kernel"] == pytest.approx(r["t_init"] + r["t_main_loop"] + r["t_epilogue"])


def test_table_rows_by_hand_two_blocks_per_cu_three_batches_batched():
    # batched Q.K^T: 96 x (512 x 64 . 64 x 512), B stored N x K, fp16 out; 128x128x64 tile,
    # 64x64 waves, S=2, R=2, fused.  16 tiles per matrix, 1536 blocks.
    d = pm.Device()
    r = pm.predict(512, 512, 64, 96, 2, 128, 128, 64, 64, 64, 2, 2, True, d, transB=True)
    # scheduler: ring 2 * 32 KiB = 64 KiB -> floor(160/64) = 2 blocks by LDS; registers
    # 64*64/64 + 2*(2+2)*4 + 48 = 144 per lane -> floor(512/144) = 3 waves per pipe -> 3 blocks
    # of 4 waves; 1536 blocks exist -> 2 per CU, 512 per batch, ceil(1536/512) = 3 batches
    assert r["n_blk_per_cu"] == 2 and r["n_threadblk_batch"] == 3
    # compute: 8 waves on 4 pipes -> all busy, one block gets half a CU
    assert r["util"] == 0.5
    assert r["t_compute"] == pytest.approx(2 * 128 * 128 * 16 / (d.flop_per_us_cu * 0.5))
    # register load: latency + 4 waves * (64+64)*16*2 B, two blocks share the port
    assert r["t_reg_load"] == pytest.approx(d.lat_lds + 16384 * 2 / d.bw_lds_cu)
    # inner pipeline: 4 fragments, 2 register stages, 2 waves per pipe multiplexed
    t_pipe = pm.pipeline_latency(r["t_reg_load"], r["t_compute"], 4, 2, 2)
    # LDS port: A 16 KiB read by 2 wave columns, B 16 KiB by 2 wave rows, both k-contiguous
    # (plain reads), plus the 32 KiB k-tile written; two blocks
    t_port = (32768 / d.bw_lds_cu + 32768 / d.bw_lds_cu + 32768 / d.bw_lds_cu) * 2
    t_fill = 32768 * 2 / (d.bw_llc / 256)          # two blocks share the CU's fill path
    assert r["t_smem_use"] == pytest.approx(max(t_pipe, t_port, t_fill))
    # memory: 512 blocks * 32 KiB over the LLC; DRAM working set: the 512 co-resident blocks are
    # 32 whole matrices of 16 tiles, each a 4 x 4 patch: (4*128 + 4*128) rows of 64 halves
    t_llc = d.lat_llc + 512 * 32768 / d.bw_llc
    t_dram = d.lat_dram + 32 * (4 * 128 + 4 * 128) * 64 * 2 / d.bw_dram
    assert r["t_smem_load"] == pytest.approx(max(t_llc, t_dram))
    assert r["t_init"] == pytest.approx(r["t_smem_load"] + r["t_reg_load"])
    # outer pipeline: one k-tile, 2 stages, 2 blocks per CU multiplexed
    assert r["t_main_loop"] == pytest.approx(pm.pipeline_latency(r["t_smem_load"], r["t_smem_use"], 1, 2, 2))
    # epilogue: 512 tiles of 128*128 fp16
    assert r["t_epilogue"] == pytest.approx(d.lat_dram_write + 512 * 32768 / d.bw_dram_write)
    assert r["t_threadblk"] == pytest.approx(r["t_init"] + r["t_main_loop"] + r["t_epilogue"])
    assert r["t_kernel"] == pytest.approx(3 * r["t_threadblk"])


def test_table_rows_by_hand_unfused_and_transposed_operands():
    # unfused R=2: one fragment load per k-tile is exposed on top of the pipelined inner loop
    d = pm.Device()
    args = (2048, 2048, 2048, 1, 2, 128, 128, 64, 64, 64, 3, 2)
    fused = pm.predict(*args, True, d)
    unfused = pm.predict(*args, False, d)
    t_pipe = pm.pipeline_latency(fused["t_reg_load"], fused["t_compute"], 4, 2, 1)
    t_port = 32768 / d.bw_lds_cu + 32768 / d.bw_lds_tr_cu + 32768 / d.bw_lds_cu
    # a fill path fast enough not to be the floor, so that the register-level terms show
    d = pm.Device(bw_llc=1e9)
    fused = pm.predict(*args, True, d)
    unfused = pm.predict(*args, False, d)
    assert fused["t_smem_use"] == pytest.approx(max(t_pipe, t_port))
    assert unfused["t_smem_use"] == pytest.approx(max(t_pipe + fused["t_reg_load"], t_port))
    assert unfused["t_smem_use"] > fused["t_smem_use"]
    # R=1 has no register pipeline to refill: fusion flag irrelevant, each fragment load exposed
    r1 = pm.predict(2048, 2048, 2048, 1, 2, 128, 128, 64, 64, 64, 3, 1, False, d)
    assert r1["t_smem_use"] == pytest.approx(max((fused["t_reg_load"] + fused["t_compute"]) * 4, t_port))
    # operand layouts only enter through the port term: A stored K x M is read through the
    # transposing read, B stored N x K through the plain one
    big = pm.Device(lat_lds=0.0, flop_per_us_cu=1e12, bw_llc=1e12)     # compute, latency and fill negligible: port term rules
    ta = pm.predict(*args, True, big, transA=True)
    tb = pm.predict(*args, True, big, transB=True)
    assert ta["t_smem_use"] == pytest.approx(32768 / big.bw_lds_tr_cu + 32768 / big.bw_lds_tr_cu + 32768 / big.bw_lds_cu)
    assert tb["t_smem_use"] == pytest.approx(32768 / big.bw_lds_cu + 32768 / big.bw_lds_cu + 32768 / big.bw_lds_cu)


def test_table_rows_by_hand_convolution_with_the_patch_in_lds():
    # conv 32 x 56 x 56 x 64 -> 64, 3x3 as a GEMM 100352 x 64 x 576, fp16 out; 256x64x64 tile, 64x64
    # waves, S=3, R=2, fused; 9 taps share one input patch that stays in LDS
    d = pm.Device()
    r = pm.predict(100352, 64, 576, 1, 2, 256, 64, 64, 64, 64, 3, 2, True, d, patch_taps=9)
    plain = pm.predict(100352, 64, 576, 1, 2, 256, 64, 64, 64, 64, 3, 2, True, d)
    # a k-tile brings 256/9 rows of A and 64 columns of B, 64 deep
    stage = (256 / 9 + 64) * 64 * 2
    # LDS: 3 stages of the 8 KiB B tile + the patch (1.5 A tiles = 48 KiB) = 72 KiB -> 2 blocks per
    # CU by LDS; registers 64 + 32 + 48 = 144 -> 3; 392 blocks -> ceil(392/256) = 2 -> 2 per CU,
    # one batch of 392 blocks
    assert r["n_blk_per_cu"] == 2 and r["n_threadblk_batch"] == 1
    assert plain["n_blk_per_cu"] == 1 and plain["n_threadblk_batch"] == 2      # 3 * 40 KiB ring
    assert r["util"] == 0.5
    assert r["t_compute"] == pytest.approx(2 * 256 * 64 * 16 / (d.flop_per_us_cu * 0.5))
    assert r["t_reg_load"] == pytest.approx(d.lat_lds + 4 * (64 + 64) * 16 * 2 * 2 / d.bw_lds_cu)
    t_pipe = pm.pipeline_latency(r["t_reg_load"], r["t_compute"], 4, 2, 2)
    # port: the whole A tile is still read from LDS (by one wave column), B by 4 wave rows through
    # the transposing read; only the fetched bytes shrink
    t_port = (256 * 64 * 2 / d.bw_lds_cu + 4 * 64 * 64 * 2 / d.bw_lds_tr_cu + stage / d.bw_lds_cu) * 2
    t_fill = stage * 2 / (d.bw_llc / 256)
    assert r["t_smem_use"] == pytest.approx(max(t_pipe, t_port, t_fill))
    t_llc = d.lat_llc + 392 * stage / d.bw_llc
    # DRAM working set: 392 tiles in one column of tiles (ntn = 1): 20 x 1 patch by the
    # near-square rule (ceil(sqrt(392)) = 20 rows, then ceil(392/20) = 20 -> capped at ntn = 1)
    t_dram = d.lat_dram + (20 * 256 / 9 + 1 * 64) * 64 * 2 / d.bw_dram
    assert r["t_smem_load"] == pytest.approx(max(t_llc, t_dram))
    assert r["t_main_loop"] == pytest.approx(pm.pipeline_latency(r["t_smem_load"], r["t_smem_use"], 9, 3, 2))
    assert r["t_epilogue"] == pytest.approx(d.lat_dram_write + 392 * 256 * 64 * 2 / d.bw_dram_write)
    assert r["t_kernel"] == pytest.approx(r["t_smem_load"] + r["t_reg_load"] + r["t_main_loop"] + r["t_epilogue"])
    # the plain kernel of the same schedule fetches 9x the A rows per k-tile
    assert plain["t_smem_load"] > r["t_smem_load"]


def test_table_rows_by_hand_persistent_blocks():
    # batched Q.K^T again, 96 x (512 x 64 . 64 x 512), fp16 out, with persistent blocks: 128x128x64
    # tile, 4 consumer waves of 64x64, S=3, R=2, fused.  1536 tiles, one k-tile each.
    d = pm.Device()
    r = pm.predict(512, 512, 64, 96, 2, 128, 128, 64, 64, 64, 3, 2, True, d, transB=True, persistent=True)
    # LDS: ring 3 * 32 KiB + staging 4 waves * 32 rows * (64*4 + 16) B = 98304 + 34816 = 133120 B
    # -> one block per CU; 256 blocks walk ceil(1536/256) = 6 tiles each
    assert r["n_blk_per_cu"] == 1 and r["n_threadblk_batch"] == 1
    assert r["util"] == 1.0
    t_compute = 2 * 128 * 128 * 16 / d.flop_per_us_cu
    t_reg_load = d.lat_lds + 16384 / d.bw_lds_cu
    t_port = 32768 / d.bw_lds_cu + 32768 / d.bw_lds_cu + 32768 / d.bw_lds_cu       # B stored N x K: plain reads
    t_fill = 32768 / (d.bw_llc / 256)
    t_smem_use = max(pm.pipeline_latency(t_reg_load, t_compute, 4, 2, 1), t_port, t_fill)
    # 256 blocks stream at once
    t_llc = d.lat_llc + 256 * 32768 / d.bw_llc
    t_dram = d.lat_dram + 16 * (4 * 128 + 4 * 128) * 64 * 2 / d.bw_dram            # 16 whole matrices of 4 x 4 tiles
    t_smem_load = max(t_llc, t_dram)
    assert r["t_smem_load"] == pytest.approx(t_smem_load)
    # the stores of a tile are consumer work of its one iteration: 256 tiles of 32 KiB in flight
    t_use = t_smem_use + (256 * 32768 / d.bw_dram_write) / 1
    assert r["t_smem_use"] == pytest.approx(t_use)
    assert r["t_init"] == pytest.approx(t_smem_load + t_reg_load)
    # one loop of 6 tiles * 1 k-tile, 3 stages
    assert r["t_main_loop"] == pytest.approx(pm.pipeline_latency(t_smem_load, t_use, 6, 3, 1))
    assert r["t_kernel"] == pytest.approx(r["t_init"] + r["t_main_loop"] + d.lat_dram_write)
    # against the tile-at-a-time schedule of the same tile: the fill and the write latency are paid
    # once, not once per batch of blocks
    plain = pm.predict(512, 512, 64, 96, 2, 128, 128, 64, 64, 64, 3, 2, True, d, transB=True)
    assert r["t_kernel"] < plain["t_kernel"]
    # long reduction axis, few tiles (2048^3: one tile per block): the stores are spread over the
    # 32 iterations of the tile
    g = pm.predict(2048, 2048, 2048, 1, 2, 128, 128, 64, 64, 64, 3, 2, True, d, persistent=True)
    t_port = 32768 / d.bw_lds_cu + 32768 / d.bw_lds_tr_cu + 32768 / d.bw_lds_cu
    t_use = max(pm.pipeline_latency(t_reg_load, t_compute, 4, 2, 1), t_port, t_fill) + (256 * 32768 / d.bw_dram_write) / 32
    assert g["t_smem_use"] == pytest.approx(t_use)
    assert g["t_main_loop"] == pytest.approx(pm.pipeline_latency(g["t_smem_load"], t_use, 32, 3, 1))
    # two blocks per CU when the LDS allows: 64x64x64 tile, S=2: 2*16 KiB + 4*32*(32*4+16) = 51200 B
    h = pm.predict(512, 512, 64, 96, 2, 64, 64, 64, 32, 32, 2, 2, True, d, transB=True, persistent=True)
    assert h["n_blk_per_cu"] == 2 and h["util"] == 0.5
    assert h["t_main_loop"] == pytest.approx(pm.pipeline_latency(h["t_smem_load"], h["t_smem_use"], 12 * 1, 2, 2))


def test_bottleneck_model_by_hand_each_resource_in_turn():
    # Sec. 6.4 comparison model: max(compute, LDS traffic, DRAM traffic), each at full rate
    # 2048^3, 128x128x64, 64x64 waves: 256 blocks, 32 k-tiles of 4 register loops
    def terms(d):
        t_cmp = 256 * 32 * 4 * (2 * 128 * 128 * 16) / (256 * d.flop_per_us_cu)
        t_lds = 256 * 32 * 4 * (4 * (64 + 64) * 16 * 2) / (256 * d.bw_lds_cu)
        t_mem = (256 * 32 * (128 + 128) * 64 * 2 + 256 * 128 * 128 * 2) / d.bw_dram
        return t_cmp, t_lds, t_mem
    args = (2048, 2048, 2048, 1, 2, 128, 128, 64, 64, 64)
    for d in (pm.Device(),
              pm.Device(flop_per_us_cu=1e3),                  # compute is the bottleneck
              pm.Device(bw_lds_cu=1e2),                       # LDS traffic is
              pm.Device(bw_dram=1e3)):                        # device memory traffic is
        assert pm.bottleneck(*args, d) == pytest.approx(max(terms(d)))
    assert pm.bottleneck(*args, pm.Device(flop_per_us_cu=1e3)) == pytest.approx(terms(pm.Device(flop_per_us_cu=1e3))[0])
    assert pm.bottleneck(*args, pm.Device(bw_lds_cu=1e2)) == pytest.approx(terms(pm.Device(bw_lds_cu=1e2))[1])
    assert pm.bottleneck(*args, pm.Device(bw_dram=1e3)) == pytest.approx(terms(pm.Device(bw_dram=1e3))[2])
    # batched, ragged: blocks = ceil(1000/128) * ceil(264/64) * 3 = 8 * 5 * 3, k-tiles = ceil(520/32)
    d = pm.Device(bw_dram=1e3)
    blocks, ktiles = 8 * 5 * 3, 17
    t_mem = (blocks * ktiles * (128 + 64) * 32 * 2 + blocks * 128 * 64 * 4) / d.bw_dram
    assert pm.bottleneck(1000, 264, 520, 3, 4, 128, 64, 32, 64, 32, d) == pytest.approx(t_mem)


def test_splitk_prediction_time_by_hand():
    # 1024 x 64 output, K = 2048, 64x64x64 tile: 32 k-tiles; 16 slices requested -> 2 k-tiles each
    d = pm.Device()
    t, slices = pm.predict_splitk(1024, 64, 2048, 1, 2, 64, 64, 64, 32, 32, 4, 2, True, 16, d)
    assert slices == 16
    # the sliced problem: 16 times the blocks, K = 2 * 64, fp32 partial tiles
    sliced = pm.predict(1024, 64, 128, 16, 4, 64, 64, 64, 32, 32, 4, 2, True, d)["t_kernel"]
    # second pass: read 16 fp32 partials and write one fp16 result per output element, one
    # DRAM read latency and one write latency
    reduce_pass = d.lat_dram + d.lat_dram_write + 1024 * 64 * (4 * 16 + 2) / d.bw_dram
    assert t == pytest.approx(sliced + reduce_pass)
    # one slice: no second pass is charged (but the output is still fp32: the kernel's own)
    t1, s1 = pm.predict_splitk(1024, 64, 2048, 1, 2, 64, 64, 64, 32, 32, 4, 2, True, 1, d)
    assert s1 == 1
    assert t1 == pytest.approx(pm.predict(1024, 64, 2048, 1, 4, 64, 64, 64, 32, 32, 4, 2, True, d)["t_kernel"])
    # batched, uneven: 33 k-tiles over 4 -> 9 per slice -> 4 slices, the last one short; the
    # model charges every slice the full 9 k-tiles
    t4, s4 = pm.predict_splitk(128, 128, 33 * 64, 3, 2, 128, 128, 64, 64, 64, 3, 2, True, 4, d)
    assert s4 == 4
    want = pm.predict(128, 128, 9 * 64, 12, 4, 128, 128, 64, 64, 64, 3, 2, True, d)["t_kernel"] + \
        d.lat_dram + d.lat_dram_write + 3 * 128 * 128 * (4 * 4 + 2) / d.bw_dram
    assert t4 == pytest.approx(want)


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
                       transA=P.get("ta", False), persistent=s.variant == 2)
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
                       bool(s.fuse_inner), patch_taps=9 if s.variant == 1 else 0, persistent=s.variant == 2)
        assert us == pytest.approx(r["t_kernel"], rel=1e-12)
        if s.variant == 1:
            seen += 1
            # less traffic per k-tile than the default kernel of the same schedule
            plain = al.sched(s.bm, s.bn, s.bk, s.wm, s.wn, s.stages, s.reg_stages, s.fuse_inner)
            assert terms[5] < al.alcop_model_predict(prob, plain, 0)[1][5]
    assert any(s.variant == 2 for s in al.alcop_sched_space(prob))
    assert seen >= 6


# ---- the learned corrector (Sec. 5.3, "Analytical + ML") ----------------------------------------
def test_corrector_features_by_their_definition():
    prob = al.problem(al.OP_GEMM, 2048, 2048, 2048, al.F16, al.F16)
    s = al.sched(256, 128, 32, 128, 64, 3, 2, 1, 1, 0)
    x = al.alcop_corrector_features(prob, s)
    a0 = al.alcop_model_predict(prob, s, 0)[0]
    a1 = al.alcop_model_predict(prob, s, 1)[0]
    want = [1.0, math.log(a0), math.log(a1), math.log2(256 * 128) - 14, math.log2(32) - 6, 3 - 2, 2 - 1, 1.0,
            math.log2(4) - 2, 0.0]
    assert x == pytest.approx(want, rel=1e-12, abs=1e-12)


def test_corrector_ridge_solve_against_a_library_solver():
    import numpy as np
    rng = np.random.default_rng(7)
    D = al.CORRECTOR_DIM
    prior = np.zeros(D)
    prior[1] = 1.0
    # no trials: the prior, i.e. the analytical model itself
    assert al.alcop_corrector_fit([], []) == pytest.approx(list(prior))
    for n in (1, 3, D, 40):
        X = rng.normal(size=(n, D))
        X[:, 0] = 1.0
        w_true = rng.normal(size=D)
        t = np.exp(X @ w_true + 0.05 * rng.normal(size=n))
        got = np.array(al.alcop_corrector_fit(X.tolist(), t.tolist()))
        want = np.linalg.solve(X.T @ X + 0.3 * np.eye(D), X.T @ np.log(t) + 0.3 * prior)
        assert got == pytest.approx(want, rel=1e-9, abs=1e-9)
    # plenty of clean data: the weights that generated it are recovered (up to the shrinkage)
    X = rng.normal(size=(4000, D))
    w_true = rng.normal(size=D)
    got = np.array(al.alcop_corrector_fit(X.tolist(), np.exp(X @ w_true).tolist()))
    assert np.max(np.abs(got - w_true)) < 1e-2
    # a measurement that agrees with the analytical model leaves the prior in place
    x = [1.0, math.log(20.0)] + [0.0] * (D - 2)
    assert al.alcop_corrector_fit([x], [20.0]) == pytest.approx(list(prior), abs=1e-12)
