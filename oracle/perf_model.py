"""The paper's static performance model (Sec. 5, Table 1), restated in plain Python for the
tests - TEST INFRASTRUCTURE ONLY; shares no code with the library's C++ model.

Symbols are the paper's.  Table 1 gives the structure; the terms it leaves open are read as
follows:

  * Util(N_warp_per_threadblk, N_threadblk_per_SM): share of one CU's matrix throughput that one
    threadblock obtains = min(1, N_warp*N_blk/4) / N_blk  (4 matrix pipes per CU).
  * T_reg_load (used in Table 1 but not defined there): LAT_LDS + Bytes_one_reg_loop * N_blk / BW_LDS.
  * N_mplx of the inner (register-level) pipeline: a DELIBERATE DEVIATION from Table 1, which
    gives N_warp_per_threadblk.  Here it is the number of wavefronts sharing one matrix pipe,
    max(1, N_warp*N_blk/4): on this machine a wavefront is pinned to one of a CU's four SIMDs and
    only the wavefronts of the same SIMD can fill each other's load latency; four waves on four
    SIMDs do not multiplex at all.
  * N_threadblk_batch: ceil(blocks / (256 * N_blk_per_CU)); N_blk_per_CU limited by LDS
    (160 KB / ring bytes), by registers (512 per lane / estimated registers per wave) and by the
    number of blocks that exist.
  * Working set of a threadblock-batch: the co-resident tiles of one matrix form a near-square
    patch; every distinct row panel and column panel is fetched once per outer iteration.
  * Without inner-pipeline fusion (not modelled by the paper, which assumes the fused steady
    state) one fragment load per outer iteration is exposed when R = 2.
  * LDS port occupancy (an addition to Table 1 for this machine): T_smem_use is at least the time
    the single LDS port needs to move the fragment reads of every wave (K-contiguous operand at
    256 B/clk, N-contiguous operand through the transposing read at ~170 B/clk) plus the
    direct-to-LDS writes of one k-tile.
  * Fill path (another addition): one compute unit's L2 -> LDS path delivers bw_llc / num_cu;
    T_smem_use is at least the time that path needs for the k-tiles of the CU's blocks.  The
    pipeline criterion of Table 1 treats a load as a latency to hide and would otherwise call a
    bandwidth-bound loop compute-bound as soon as there are enough stages.
  * Clock: rates are taken at the ~1.8 GHz a GEMM sustains under the power cap.

Pins (tests/test_model.py): the pipeline latency model against hand-computed values and the
equivalence of its two printed forms (Table 1 and the captions of Fig. 7); every other row of
Table 1 against values worked out by hand for one schedule.
"""
from __future__ import annotations

import math
from dataclasses import dataclass


@dataclass
class Device:
    num_cu: int = 256
    simd_per_cu: int = 4
    lds_bytes: float = 163840.0
    regs_per_lane: float = 512.0
    flop_per_us_cu: float = 4096.0 * 1800.0      # sustained clock under the power cap ~1.8 GHz
    lat_lds: float = 128.0 / 1800.0
    bw_lds_cu: float = 256.0 * 1800.0            # ds_read_b128 and DMA writes (measured)
    bw_lds_tr_cu: float = 170.0 * 1800.0         # transposing 8-byte read (measured)
    lat_llc: float = 0.6
    bw_llc: float = 40.0 * 256.0 * 1800.0        # 40 B/clk per CU when all CUs stream (measured)
    lat_dram: float = 1.2
    bw_dram: float = 8.0e6
    lat_dram_write: float = 1.0
    bw_dram_write: float = 8.0e6


def pipeline_latency(t_load, t_use, n_loop, n_pipe, n_mplx):
    """Table 1, 'Pipeline Latency Model'."""
    if t_load <= (n_pipe * n_mplx - 1) * t_use:
        return t_use * n_loop
    return (t_load + t_use) * n_loop / n_pipe


def pipeline_latency_caption_form(t_load, t_use, n_loop, n_pipe, n_mplx):
    """The same criterion as printed under Fig. 7: case 1 iff t_use*N_mplx*N_pipe >= t_load + t_use."""
    if t_use * n_mplx * n_pipe >= t_load + t_use:
        return t_use * n_loop
    return (t_load + t_use) * n_loop / n_pipe


def predict(M, N, K, batch, out_bytes, bm, bn, bk, wm, wn, S, R, fuse, dev: Device = Device(),
            transB: bool = False, transA: bool = False, patch_taps: int = 0, persistent: bool = False):
    """Returns a dict of the Table 1 quantities (microseconds).

    patch_taps > 0 (not in the paper): a convolution whose input patch stays in LDS; the A rows
    of a tile are fetched once per block instead of once per filter tap, so one k-tile accounts
    for bm / patch_taps of them, and the patch (reading: 1.5 tiles) occupies LDS beside the
    ring of B tiles.

    persistent (not in the paper): blocks that stay on their compute unit and walk a list of
    tiles; a block's tiles form one load-and-use loop, the epilogue's stores are consumer work
    inside that loop (bandwidth term only, they are not waited for), T_init is paid once and
    one write latency ends the kernel.  A staging band per consumer wave follows the ring in
    LDS, and at most two blocks share a compute unit."""
    ntm, ntn = math.ceil(M / bm), math.ceil(N / bn)
    tiles = ntm * ntn
    n_blocks = tiles * batch
    n_warp = (bm // wm) * (bn // wn)
    n_smem_loop = math.ceil(K / bk)
    n_reg_loop = bk // 16
    a_rows = bm / patch_taps if patch_taps > 0 else bm
    bytes_one_smem_loop = (a_rows + bn) * bk * 2
    lds_use = (S * bn * bk * 2 + 1.5 * bm * bk * 2) if patch_taps > 0 else S * bytes_one_smem_loop
    if persistent:
        lds_use += n_warp * 32 * (wn * 4 + 16)
    bytes_one_reg_loop = n_warp * (wm + wn) * 16 * 2
    flops_one_reg_loop = 2 * bm * bn * 16

    # simulated scheduler
    regs = wm * wn / 64 + R * (wm / 32 + wn / 32) * 4 + 48
    waves_per_simd = max(1, min(8, math.floor(dev.regs_per_lane / regs)))
    n_blk_per_cu = min(math.floor(dev.lds_bytes / lds_use),
                       math.floor(waves_per_simd * dev.simd_per_cu / n_warp))
    n_blk_per_cu = max(1, n_blk_per_cu)
    if persistent:
        n_blk_per_cu = max(1, min(2, math.floor(dev.lds_bytes / lds_use)))
    n_blk_per_cu = min(n_blk_per_cu, math.ceil(n_blocks / dev.num_cu))
    n_batch = math.ceil(n_blocks / (dev.num_cu * n_blk_per_cu))
    n_blk_per_batch = min(n_blocks, dev.num_cu * n_blk_per_cu)

    # Computation Latency Model
    util = min(1.0, n_warp * n_blk_per_cu / dev.simd_per_cu) / n_blk_per_cu
    t_compute = flops_one_reg_loop / (dev.flop_per_us_cu * util)

    # Threadblock Latency Model, inner level
    t_reg_load = dev.lat_lds + bytes_one_reg_loop * n_blk_per_cu / dev.bw_lds_cu
    n_mplx_inner = max(1.0, n_warp * n_blk_per_cu / dev.simd_per_cu)
    t_smem_use = pipeline_latency(t_reg_load, t_compute, n_reg_loop, R, n_mplx_inner)
    if not fuse and R >= 2:
        t_smem_use += t_reg_load
    # LDS port occupancy: fragment reads of all waves + DMA writes of the next k-tile share one port
    a_read = bm * bk * 2 * (bn // wn)
    b_read = bn * bk * 2 * (bm // wm)
    t_port = (a_read / (dev.bw_lds_tr_cu if transA else dev.bw_lds_cu) + b_read / (dev.bw_lds_cu if transB else dev.bw_lds_tr_cu)
              + bytes_one_smem_loop / dev.bw_lds_cu) * n_blk_per_cu
    t_smem_use = max(t_smem_use, t_port)
    # fill path of one compute unit: its blocks cannot consume k-tiles faster than L2 -> LDS delivers
    t_fill = bytes_one_smem_loop * n_blk_per_cu / (dev.bw_llc / dev.num_cu)
    t_smem_use = max(t_smem_use, t_fill)

    # Memory Latency Model
    t_llc_load = dev.lat_llc + bytes_one_smem_loop * n_blk_per_batch / dev.bw_llc
    per_mat = min(tiles, n_blk_per_batch)
    mats = math.ceil(n_blk_per_batch / tiles)
    rows_u = min(ntm, math.ceil(math.sqrt(per_mat)))
    cols_u = min(ntn, math.ceil(per_mat / rows_u))
    workset = (rows_u * a_rows + cols_u * bn) * bk * 2 * mats
    t_dram_load = dev.lat_dram + workset / dev.bw_dram
    t_smem_load = max(t_llc_load, t_dram_load)

    t_init = t_smem_load + t_reg_load
    if persistent:
        tiles_per_block = math.ceil(n_blocks / (dev.num_cu * n_blk_per_cu))
        t_store = bm * bn * out_bytes * n_blk_per_batch / dev.bw_dram_write
        t_use = t_smem_use + t_store / n_smem_loop
        t_main_loop = pipeline_latency(t_smem_load, t_use, tiles_per_block * n_smem_loop, S, n_blk_per_cu)
        t_kernel = t_init + t_main_loop + dev.lat_dram_write
        return dict(t_kernel=t_kernel, t_threadblk=t_kernel, t_init=t_init, t_main_loop=t_main_loop,
                    t_epilogue=dev.lat_dram_write, t_smem_load=t_smem_load, t_smem_use=t_use,
                    n_threadblk_batch=1, t_compute=t_compute, t_reg_load=t_reg_load,
                    n_blk_per_cu=n_blk_per_cu, util=util)
    t_main_loop = pipeline_latency(t_smem_load, t_smem_use, n_smem_loop, S, n_blk_per_cu)
    # Epilogue Model
    t_epilogue = dev.lat_dram_write + bm * bn * out_bytes * n_blk_per_batch / dev.bw_dram_write
    t_threadblk = t_init + t_main_loop + t_epilogue
    t_kernel = t_threadblk * n_batch
    return dict(t_kernel=t_kernel, t_threadblk=t_threadblk, t_init=t_init, t_main_loop=t_main_loop,
                t_epilogue=t_epilogue, t_smem_load=t_smem_load, t_smem_use=t_smem_use,
                n_threadblk_batch=n_batch, t_compute=t_compute, t_reg_load=t_reg_load,
                n_blk_per_cu=n_blk_per_cu, util=util)


def bottleneck(M, N, K, batch, out_bytes, bm, bn, bk, wm, wn, dev: Device = Device()):
    """The bottleneck-only comparison model of Sec. 6.4: max of compute, LDS traffic and device
    memory traffic, each at full rate, no latency and no occupancy effects."""
    n_blocks = math.ceil(M / bm) * math.ceil(N / bn) * batch
    n_warp = (bm // wm) * (bn // wn)
    steps = math.ceil(K / bk) * (bk // 16)
    t_cmp = n_blocks * steps * 2 * bm * bn * 16 / (dev.num_cu * dev.flop_per_us_cu)
    t_lds = n_blocks * steps * n_warp * (wm + wn) * 16 * 2 / (dev.num_cu * dev.bw_lds_cu)
    t_mem = (n_blocks * math.ceil(K / bk) * (bm + bn) * bk * 2 + n_blocks * bm * bn * out_bytes) / dev.bw_dram
    return max(t_cmp, t_lds, t_mem)


def predict_splitk(M, N, K, batch, out_bytes, bm, bn, bk, wm, wn, S, R, fuse, split,
                   dev: Device = Device(), transB: bool = False):
    """Split-K schedule (not in the paper; its model applied to the sliced problem): the
    reduction axis is cut into slices of whole k-tiles, each slice is a block of its own writing
    an fp32 partial tile, and a second pass adds the slices.  `split` slices are requested; the
    k-tiles are dealt evenly, so fewer may result.  Returns (microseconds, slices)."""
    n_tiles_k = math.ceil(K / bk)
    per = math.ceil(n_tiles_k / split)
    slices = math.ceil(n_tiles_k / per)
    t = predict(M, N, per * bk, batch * slices, 4, bm, bn, bk, wm, wn, S, R, fuse, dev,
                transB=transB)["t_kernel"]
    if slices > 1:
        t += dev.lat_dram + dev.lat_dram_write + batch * M * N * (4.0 * slices + out_bytes) / dev.bw_dram
    return t, slices
