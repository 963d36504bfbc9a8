"""The kernel template itself, run on the CPU.

tests/emu builds the product's host code and kernel header against a functional model of the
gfx950 operations the loop uses (one fibre per lane).  These tests compare its results with the
oracle bit for bit on integer data, under timing policies chosen to expose a missing wait or
barrier, and require that no access left the operands or the block's LDS.  They also plant
synchronisation mistakes in the model to show that the checks would notice one.  No GPU is
involved: what this proves is the kernel's indexing, bounds and synchronisation logic, not its
speed."""
import numpy as np
import pytest
import torch

import emu_util as emu
import oracle
import paper_2210_16691_amd as al
import workloads as wl

TDT = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}
ODT = {"f16": oracle.F16, "bf16": oracle.BF16}
ADT = {"f16": al.F16, "bf16": al.BF16, "f32": al.F32}


def _exact(C, ref):
    return np.array_equal(C.double().numpy(), ref)


# ---- the model's own arithmetic, pinned against numpy / torch -------------------------------
def test_model_number_conversions():
    L = emu.lib()
    h = np.arange(65536, dtype=np.uint16)
    want = h.view(np.float16).astype(np.float32)
    got = np.array([L.emu_f16_to_f32(int(v)) for v in h], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32)[~np.isnan(want)], want.view(np.uint32)[~np.isnan(want)])
    assert np.isnan(got[np.isnan(want)]).all()
    # fp32 -> fp16, round to nearest even: every fp16 value, every midpoint between neighbours,
    # values just off the midpoints, the overflow threshold, and random numbers
    fin = want[np.isfinite(want)]
    fin = np.unique(fin)
    mids = ((fin[:-1].astype(np.float64) + fin[1:].astype(np.float64)) / 2).astype(np.float32)
    rng = np.random.default_rng(5)
    rnd = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 12, 20000))).astype(np.float32)
    xs = np.concatenate([fin, mids, np.nextafter(mids, np.float32(np.inf)), np.nextafter(mids, np.float32(-np.inf)),
                         np.float32([65504, 65519.9, 65520, 65536, 1e9, -65520, 2.0 ** -25, 2.0 ** -24, 0.0, -0.0]),
                         rnd])
    with np.errstate(over="ignore"):
        want16 = xs.astype(np.float16).view(np.uint16)
    got16 = np.array([L.emu_f32_to_f16(float(v)) for v in xs], dtype=np.uint16)
    assert np.array_equal(got16, want16)
    t = torch.from_numpy(rnd)
    want_bf = t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got_bf = np.array([L.emu_f32_to_bf16(float(v)) for v in rnd], dtype=np.uint16)
    assert np.array_equal(got_bf, want_bf)


# ---- GEMM: every emulated schedule, every layout, ragged edges ------------------------------
def _gemm_case(dt, transA, transB, s, M, N, K, policy, out="f16", seed=0, mutation=0):
    A = wl.small_ints((K, M) if transA else (M, K), dt, 900 + seed)
    B = wl.small_ints((N, K) if transB else (K, N), dt, 901 + seed)
    C = torch.full((M, N), float("nan"), dtype=TDT[out])
    errs = emu.call(al.alcop_gemm, A, B, C, s, transB=bool(transB), transA=bool(transA),
                    reads=[A, B], writes=[C], policy=policy, mutation=mutation)
    ref = oracle.gemm(wl.bits(A.t().contiguous() if transA else A),
                      wl.bits(B.t().contiguous() if transB else B), ODT[dt])
    return errs, _exact(C, ref)


@pytest.mark.parametrize("dt,transA,transB", [("f16", 0, 0), ("f16", 0, 1), ("f16", 1, 0), ("f16", 1, 1),
                                               ("bf16", 0, 0), ("bf16", 0, 1), ("bf16", 1, 1)])
def test_gemm_exact_and_in_bounds_every_emulated_schedule(dt, transA, transB):
    prob = al.problem(al.OP_GEMM, 512, 512, 512, ADT[dt], ADT[dt], transB=bool(transB), transA=bool(transA))
    scheds = emu.space(prob, opt_in=True)          # includes the k-tile-128 kernels
    assert scheds
    for n, s in enumerate(scheds):
        # two row tiles (the second ragged), a ragged column tile, three k-tiles and a partial one
        M = s.bm + 40
        N = s.bn - 24 if s.bn > 64 else 64 + 8
        K = 3 * s.bk + 8
        for policy in (emu.POLICIES[n % 4], emu.POLICIES[(n + 1) % 4]):
            errs, ok = _gemm_case(dt, transA, transB, s, M, N, K, policy, seed=n)
            assert not errs, (repr(s), policy, errs[:4])
            assert ok, (repr(s), policy)


def test_gemm_all_timing_policies_many_k_tiles_and_fp32_output():
    # more k-tiles than ring slots, so that every slot is refilled several times
    for s in (al.sched(128, 128, 64, 64, 64, 4, 2, 1), al.sched(128, 128, 64, 64, 64, 3, 1, 0),
              al.sched(64, 64, 32, 32, 32, 4, 2, 1)):
        for policy in emu.POLICIES:
            errs, ok = _gemm_case("f16", 0, 0, s, 2 * s.bm, s.bn, 11 * s.bk, policy, out="f32")
            assert not errs and ok, (repr(s), policy, errs[:4])


def test_deep_register_pipeline_every_k_tile_count_and_policy():
    # R - 1 fragments in flight: the reads run up to a whole k-tile ahead of the matrix
    # instructions and the synchronisation sits in the middle of a k-tile.  One k-tile (the
    # pipeline never reaches its steady state), two, one more than the ring holds, many; a
    # partial last k-tile; R = 3 on four fragments (body of three k-tiles) and on two
    # fragments (all of a k-tile in flight); R = 4 on four and on eight fragments.
    for s in (al.sched(128, 128, 64, 64, 64, 4, 4, 1), al.sched(128, 128, 64, 64, 64, 2, 3, 1),
              al.sched(128, 128, 32, 64, 64, 3, 3, 1), al.sched(128, 128, 128, 64, 64, 2, 4, 1),
              al.sched(64, 64, 64, 32, 32, 3, 4, 1)):
        for nk, extra in ((1, 0), (2, 0), (s.stages + 1, 8), (7, 0), (11, 16)):
            for policy in emu.POLICIES:
                errs, ok = _gemm_case("f16", 0, 0, s, s.bm + 8, s.bn, nk * s.bk + extra, policy, out="f32")
                assert not errs and ok, (repr(s), nk, extra, policy, errs[:4])
    errs, ok = _gemm_case("f16", 0, 0, al.sched(128, 128, 64, 64, 64, 4, 4, 1), 8, 8, 8, (1, 1))
    assert not errs and ok


def test_deep_register_pipeline_convolution_and_splitk():
    x = wl.small_ints((2, 9, 7, 64), "f16", 31)
    w = wl.small_ints((3, 3, 64, 64), "f16", 32)
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (1, 1), (1, 1))
    for s in (al.sched(128, 64, 64, 64, 32, 3, 4, 1), al.sched(256, 64, 64, 64, 64, 3, 4, 1, 1, 0, 1)):
        for policy in ((1, 0), (0, 1)):
            y = torch.full((2, 9, 7, 64), float("nan"), dtype=torch.float32)
            errs = emu.call(al.alcop_conv2d_igemm, x, w, y, (1, 1), (1, 1), s, reads=[x, w], writes=[y],
                            policy=policy)
            assert not errs, (repr(s), errs[:4])
            assert _exact(y, ref), repr(s)
    A = wl.small_ints((136, 7 * 64), "f16", 33)
    B = wl.small_ints((7 * 64, 72), "f16", 34)
    ref = oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16)
    C = torch.full((136, 72), float("nan"), dtype=torch.float32)
    ws = torch.empty(al.alcop_splitk_workspace_bytes(1, 136, 72, 3) // 4, dtype=torch.float32)
    errs = emu.call(al.alcop_gemm_splitk, A, B, C, 3, ws, al.sched(128, 128, 64, 64, 64, 3, 4, 1),
                    reads=[A, B], writes=[C, ws], policy=(1, 1))
    assert not errs, errs[:4]
    assert _exact(C, ref)


def test_gemm_tiny_and_single_k_tile():
    s = al.sched(64, 64, 32, 32, 32, 4, 2, 1)
    for (M, N, K) in ((1, 8, 8), (8, 8, 32), (64, 64, 16), (65, 72, 40)):
        errs, ok = _gemm_case("f16", 0, 0, s, M, N, K, (1, 0))
        assert not errs and ok, (M, N, K, errs[:4])


def test_l2_touches_stay_inside_the_operands():
    # the third (HBM -> L2) level reads ahead with plain global loads: several tiles in both
    # directions, ragged edges, more k-tiles than the look-ahead, both layouts of B
    for transB in (0, 1):
        s = al.sched(128, 128, 64, 64, 64, 4, 2, 1, 1, 4)
        errs, ok = _gemm_case("f16", 0, transB, s, 3 * 128 - 56, 2 * 128 + 8, 7 * 64, (1, 0))
        assert not errs and ok, (transB, errs[:4])
    s = al.sched(64, 64, 32, 32, 32, 4, 2, 1, 1, 8)
    errs, ok = _gemm_case("f16", 0, 0, s, 5 * 64, 3 * 64, 3 * 32, (0, 1))     # look-ahead > k-tiles
    assert not errs and ok, errs[:4]
    errs, ok = _gemm_case("f16", 0, 0, s, 5 * 64 - 8, 3 * 64 - 8, 5 * 32 + 8, (1, 1))   # partial k-tile: level off
    assert not errs and ok, errs[:4]


def test_leading_dimensions_and_output_guard():
    # operands and output are views into larger arrays; only the views are registered, so a read
    # or store one element outside them is an error
    s = al.sched(128, 128, 32, 64, 64, 3, 2, 1)
    M, N, K = 136, 200, 72
    Abig = wl.small_ints((M, K + 24), "f16", 1)
    Bbig = wl.small_ints((K, N + 16), "f16", 2)
    Cbig = torch.full((M, N + 8), float("nan"), dtype=torch.float16)
    A, B, C = Abig[:, :K], Bbig[:, :N], Cbig[:, :N]
    errs = emu.call(al.alcop_gemm, A, B, C, s, reads=[A, B], writes=[C], policy=(1, 1))
    assert not errs, errs[:4]
    ref = oracle.gemm(wl.bits(A.contiguous()), wl.bits(B.contiguous()), oracle.F16)
    assert _exact(C, ref)
    assert torch.isnan(Cbig[:, N:]).all()


# ---- fused epilogue, BMM, convolution ---------------------------------------------------------
def test_fused_epilogue_and_bmm():
    s = al.sched(128, 128, 64, 64, 64, 3, 2, 1)
    M, N, K = 136, 72, 136
    A = wl.small_ints((M, K), "f16", 11)
    B = wl.small_ints((K, N), "f16", 12)
    bias = torch.arange(N, dtype=torch.float32) - 30
    C = torch.full((M, N), float("nan"), dtype=torch.float32)
    errs = emu.call(al.alcop_gemm_fused, A, B, C, 0.5, bias, 1, s, reads=[A, B, bias], writes=[C])
    assert not errs, errs[:4]
    ref = oracle.epilogue(oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16), 0.5, bias.double().numpy(), 1)
    assert _exact(C, ref)
    # batched, B stored N x K, batch strides of views
    b = 3
    Q = wl.small_ints((b, 72, 64), "f16", 13)
    Kt = wl.small_ints((b + 1, 136, 64), "f16", 14)[1:]
    P = torch.full((b, 72, 136), float("nan"), dtype=torch.float16)
    for policy in ((1, 0), (0, 1)):
        errs = emu.call(al.alcop_bmm, Q, Kt, P, al.sched(64, 64, 64, 32, 32, 3, 2, 1), transB=True,
                        reads=[Q, Kt], writes=[P], policy=policy)
        assert not errs, errs[:4]
        ref = oracle.bmm(wl.bits(Q), wl.bits(Kt.contiguous().transpose(1, 2).contiguous()), oracle.F16)
        assert _exact(P, ref)


@pytest.mark.parametrize("geom", [
    dict(N=2, H=9, W=7, C=64, K=64, R=3, S=3, stride=(1, 1), pad=(1, 1)),
    dict(N=1, H=12, W=10, C=32, K=72, R=3, S=3, stride=(2, 2), pad=(1, 1)),
    dict(N=3, H=6, W=6, C=64, K=64, R=1, S=1, stride=(1, 1), pad=(0, 0)),
    dict(N=1, H=8, W=8, C=64, K=128, R=5, S=3, stride=(1, 2), pad=(2, 0)),
])
def test_conv_gather_exact_and_in_bounds(geom):
    g = geom
    x = wl.small_ints((g["N"], g["H"], g["W"], g["C"]), "f16", 21)
    w = wl.small_ints((g["R"], g["S"], g["C"], g["K"]), "f16", 22)
    P = (g["H"] + 2 * g["pad"][0] - g["R"]) // g["stride"][0] + 1
    Q = (g["W"] + 2 * g["pad"][1] - g["S"]) // g["stride"][1] + 1
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, g["stride"], g["pad"])
    prob = al.problem(al.OP_CONV2D, g["N"] * P * Q, g["K"], g["R"] * g["S"] * g["C"], al.F16, al.F16,
                      conv_C=g["C"])
    scheds = emu.space(prob)
    assert len(scheds) >= 2
    for n, s in enumerate(scheds):
        y = torch.full((g["N"], P, Q, g["K"]), float("nan"), dtype=torch.float16)
        errs = emu.call(al.alcop_conv2d_igemm, x, w, y, g["stride"], g["pad"], s,
                        reads=[x, w], writes=[y], policy=emu.POLICIES[n % 4])
        assert not errs, (repr(s), errs[:4])
        assert _exact(y, ref), repr(s)


# ---- the checks notice planted mistakes ------------------------------------------------------------
def test_planted_synchronisation_mistakes_are_noticed():
    s4 = al.sched(128, 128, 64, 64, 64, 4, 2, 1)
    s3u = al.sched(128, 128, 64, 64, 64, 3, 1, 0)
    s4d = al.sched(128, 128, 64, 64, 64, 4, 4, 1)       # three fragments in flight
    M, N, K = 128, 128, 8 * 64
    # sound kernel: clean under every policy (the control)
    for s in (s4, s3u, s4d):
        for policy in emu.POLICIES:
            errs, ok = _gemm_case("f16", 0, 0, s, M, N, K, policy)
            assert not errs and ok
    # a wait that lets too many loads stay in flight: a late-landing load is read too early
    for s in (s4, s3u, s4d):
        errs, ok = _gemm_case("f16", 0, 0, s, M, N, K, (1, 0), mutation=1)
        assert not ok, repr(s)
    # no block barrier: a wave that runs ahead reads tiles the others have not delivered, or
    # refills a slot the others still read
    for s in (s4, s4d):
        for policy in ((0, 0), (0, 1), (1, 0)):
            errs, ok = _gemm_case("f16", 0, 0, s, M, N, K, policy, mutation=2)
            assert not ok, (repr(s), policy)
    # waits ignored altogether
    for s in (s4, s4d):
        errs, ok = _gemm_case("f16", 0, 0, s, M, N, K, (1, 0), mutation=3)
        assert not ok, repr(s)
    # no wait for the LDS reads before the barrier that releases a slot: the refill may overtake
    # a read (the data path of the model cannot show this, the in-flight bookkeeping does)
    for s in (s4, s3u, s4d, al.sched(128, 128, 64, 64, 64, 1, 1, 0)):
        errs, ok = _gemm_case("f16", 0, 0, s, M, N, K, (1, 0), mutation=4)
        assert errs and "may still be fetching" in " ".join(errs), repr(s)


def test_out_of_bounds_accesses_are_noticed():
    # the same correct call, but the test "forgets" the last row of A / the last row of C when it
    # declares the operands: the model must report the accesses that leave the declared ranges
    s = al.sched(128, 128, 64, 64, 64, 2, 2, 1)
    A = wl.small_ints((128, 128), "f16", 31)
    B = wl.small_ints((128, 128), "f16", 32)
    C = torch.zeros(128, 128, dtype=torch.float16)
    assert not emu.call(al.alcop_gemm, A, B, C, s, reads=[A, B], writes=[C])
    errs = emu.call(al.alcop_gemm, A, B, C, s, reads=[A[:127], B], writes=[C])
    assert errs and "descriptor admits" in " ".join(errs)
    errs = emu.call(al.alcop_gemm, A, B, C, s, reads=[A, B], writes=[C[:127]])
    assert errs and "global store outside" in " ".join(errs)
    errs = emu.call(al.alcop_gemm, A, B, C, s, reads=[A, B, C], writes=[])
    assert errs      # C declared read-only


# ---- split-K ---------------------------------------------------------------------------------------
def _ws(batch, M, N, split):
    n = al.alcop_splitk_workspace_bytes(batch, M, N, split)
    assert n == 4 * split * batch * M * N
    return torch.full((n // 4,), float("nan"), dtype=torch.float32)


@pytest.mark.parametrize("transB", [0, 1])
def test_splitk_gemm_exact_in_bounds_every_emulated_variant(transB):
    dt = "f16"
    scheds = [al.sched(128, 128, 64, 64, 64, 3, 2, 1), al.sched(64, 64, 64, 32, 32, 2 if transB else 4, 2, 1)]
    if not transB:
        scheds.append(al.sched(128, 128, 64, 64, 64, 1, 1, 0))
    for n, s in enumerate(scheds):
        # ragged M and N, 9 k-tiles and a partial one: slices of unequal length, the last one short
        M, N, K = s.bm + 24, s.bn + 8, 9 * 64 + 24
        A = wl.small_ints((M, K), dt, 40 + n)
        B = wl.small_ints((N, K) if transB else (K, N), dt, 41 + n)
        ref = oracle.gemm(wl.bits(A), wl.bits(B.t().contiguous() if transB else B), ODT[dt])
        for split in (2, 4, 7, 10, 64):
            C = torch.full((M, N), float("nan"), dtype=torch.float16)
            ws = _ws(1, M, N, split)
            errs = emu.call(al.alcop_gemm_splitk, A, B, C, split, ws, s, transB=bool(transB),
                            reads=[A, B], writes=[C, ws], policy=emu.POLICIES[(n + split) % 4])
            assert not errs, (repr(s), split, errs[:4])
            assert _exact(C, ref), (repr(s), split)


def test_splitk_fused_epilogue_batched_bf16_and_auto():
    b, M, N, K = 2, 72, 136, 5 * 64
    A = wl.small_ints((b, M, K), "bf16", 51)
    B = wl.small_ints((b, K, N), "bf16", 52)
    bias = (torch.arange(N, dtype=torch.float32) % 7) - 3
    C = torch.full((b, M, N), float("nan"), dtype=torch.float32)
    s = al.sched(128, 128, 64, 64, 64, 2, 2, 1)
    ws = _ws(b, M, N, 3)
    errs = emu.call(al.alcop_gemm_splitk, A, B, C, 3, ws, s, 0.25, bias, 1,
                    reads=[A, B, bias], writes=[C, ws], policy=(0, 1))
    assert not errs, errs[:4]
    ref = oracle.epilogue(oracle.bmm(wl.bits(A), wl.bits(B), oracle.BF16), 0.25, bias.double().numpy(), 1)
    assert _exact(C, ref)
    # the model's pick for a small output with a long reduction axis uses several slices and is
    # predicted faster than the best unsplit schedule; too small a workspace is refused
    with emu._swapped():
        prob = al.problem(al.OP_GEMM, 128, 64, 4096, al.F16, al.F16)
        s2, split, us = al.alcop_splitk_auto(prob)
        assert split > 1
        assert us < al.alcop_model_predict(prob, al.alcop_sched_auto(prob), 0)[0]
        assert al.alcop_splitk_auto(prob, 4)[1] == 4
    A2 = wl.small_ints((128, 512), "f16", 53)
    B2 = wl.small_ints((512, 64), "f16", 54)
    C2 = torch.zeros(128, 64, dtype=torch.float16)
    small = torch.zeros(128 * 64 * 4 - 1, dtype=torch.float32)
    with pytest.raises(al.AlcopError) as e:
        emu.call(al.alcop_gemm_splitk, A2, B2, C2, 4, small, None, reads=[A2, B2], writes=[C2, small])
    assert e.value.code == al.ERR_SIZE
    # automatic schedule and split on the emulator's own table
    ws2 = _ws(1, 128, 64, 64)
    errs = emu.call(al.alcop_gemm_splitk, A2, B2, C2, 0, ws2, None, reads=[A2, B2], writes=[C2, ws2])
    assert not errs, errs[:4]
    assert _exact(C2, oracle.gemm(wl.bits(A2), wl.bits(B2), oracle.F16))


def test_splitk_conv_exact_and_in_bounds():
    g = dict(N=1, H=7, W=9, C=128, K=72, R=3, S=3, stride=(1, 1), pad=(1, 1))
    x = wl.small_ints((g["N"], g["H"], g["W"], g["C"]), "f16", 61)
    w = wl.small_ints((g["R"], g["S"], g["C"], g["K"]), "f16", 62)
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, g["stride"], g["pad"])
    M = g["N"] * g["H"] * g["W"]
    for n, s in enumerate((al.sched(128, 64, 64, 64, 32, 3, 2, 1), al.sched(64, 64, 64, 32, 32, 1, 1, 0),
                           al.sched(64, 128, 64, 32, 64, 4, 2, 1))):
        for split in (2, 3, 5, 18):       # 18 k-tiles of 64: slices start inside taps and at taps
            y = torch.full((g["N"], g["H"], g["W"], g["K"]), float("nan"), dtype=torch.float16)
            ws = _ws(1, M, g["K"], split)
            errs = emu.call(al.alcop_conv2d_igemm_splitk, x, w, y, split, ws, g["stride"], g["pad"], s,
                            reads=[x, w], writes=[y, ws], policy=emu.POLICIES[(n + split) % 4])
            assert not errs, (repr(s), split, errs[:4])
            assert _exact(y, ref), (repr(s), split)


# ---- convolution with KRSC weights -------------------------------------------------------------
@pytest.mark.parametrize("geom", [
    dict(N=2, H=9, W=7, C=64, K=72, R=3, S=3, stride=(1, 1), pad=(1, 1)),
    dict(N=1, H=12, W=10, C=32, K=64, R=3, S=2, stride=(2, 1), pad=(1, 0)),
])
def test_conv_krsc_weights_exact_and_in_bounds(geom):
    g = geom
    x = wl.small_ints((g["N"], g["H"], g["W"], g["C"]), "f16", 71)
    w = wl.small_ints((g["R"], g["S"], g["C"], g["K"]), "f16", 72)
    wk = w.permute(3, 0, 1, 2).contiguous()                  # [K][R][S][C]
    P = (g["H"] + 2 * g["pad"][0] - g["R"]) // g["stride"][0] + 1
    Q = (g["W"] + 2 * g["pad"][1] - g["S"]) // g["stride"][1] + 1
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, g["stride"], g["pad"])
    prob = al.problem(al.OP_CONV2D, g["N"] * P * Q, g["K"], g["R"] * g["S"] * g["C"], al.F16, al.F16,
                      conv_C=g["C"], transB=True)
    scheds = emu.space(prob)
    assert scheds
    for n, s in enumerate(scheds):
        y = torch.full((g["N"], P, Q, g["K"]), float("nan"), dtype=torch.float16)
        errs = emu.call(al.alcop_conv2d_igemm_krsc, x, wk, y, g["stride"], g["pad"], s,
                        reads=[x, wk], writes=[y], policy=emu.POLICIES[n % 4])
        assert not errs, (repr(s), errs[:4])
        assert _exact(y, ref), repr(s)


# ---- block -> tile mapping, batched transposed layouts, bf16 convolution -------------------------
@pytest.mark.parametrize("ntm,ntn,raster", [(4, 4, 1), (10, 4, 1), (9, 3, 1), (3, 8, 1), (5, 4, 0), (16, 1, 1)])
def test_every_tile_is_computed_exactly_once(ntm, ntn, raster):
    # tile counts that are / are not a multiple of 8 (the XCD-aware renumbering), more row tiles
    # than one group of 8, a ragged last group; C starts as NaN, so a tile nobody computes shows
    s = al.sched(64, 64, 32, 32, 32, 2, 1, 0, raster)
    M, N, K = ntm * 64 - 8, ntn * 64 - 16, 64
    errs, ok = _gemm_case("bf16", 0, 0, s, M, N, K, (0, 0), out="f32", seed=ntm * 10 + ntn)
    assert not errs and ok, errs[:4]


def test_batched_with_a_stored_k_by_m_and_b_stored_n_by_k():
    b, M, N, K = 2, 136, 72, 96
    A = wl.small_ints((b, K, M), "f16", 81)
    B = wl.small_ints((b, N, K), "f16", 82)
    C = torch.full((b, M, N), float("nan"), dtype=torch.float16)
    s = al.sched(128, 128, 64, 64, 64, 3, 2, 1)
    errs = emu.call(al.alcop_bmm, A, B, C, s, transB=True, transA=True, reads=[A, B], writes=[C], policy=(1, 1))
    assert not errs, errs[:4]
    ref = oracle.bmm(wl.bits(A.transpose(1, 2).contiguous()), wl.bits(B.transpose(1, 2).contiguous()), oracle.F16)
    assert _exact(C, ref)


def test_bf16_convolution_with_fp32_output():
    x = wl.small_ints((2, 6, 5, 64), "bf16", 91)
    w = wl.small_ints((3, 3, 64, 64), "bf16", 92)
    y = torch.full((2, 6, 5, 64), float("nan"), dtype=torch.float32)
    errs = emu.call(al.alcop_conv2d_igemm, x, w, y, (1, 1), (1, 1), al.sched(128, 64, 64, 64, 32, 3, 2, 1),
                    reads=[x, w], writes=[y], policy=(1, 0))
    assert not errs, errs[:4]
    assert _exact(y, oracle.conv2d(wl.bits(x), wl.bits(w), oracle.BF16, (1, 1), (1, 1)))


# ---- convolution with channel counts the k-tile does not divide -----------------------------------
@pytest.mark.parametrize("geom", [
    dict(N=1, H=14, W=12, C=8, K=64, R=7, S=7, stride=(2, 2), pad=(3, 3)),     # padded RGB stem
    dict(N=2, H=7, W=6, C=24, K=72, R=3, S=3, stride=(1, 1), pad=(1, 1)),
    dict(N=1, H=6, W=9, C=40, K=64, R=3, S=2, stride=(1, 2), pad=(0, 1)),
    dict(N=1, H=5, W=5, C=96, K=64, R=1, S=1, stride=(1, 1), pad=(0, 0)),      # bk = 64 does not divide 96
    dict(N=1, H=6, W=6, C=16, K=64, R=5, S=5, stride=(1, 1), pad=(2, 2)),
])
def test_conv_any_channel_multiple_of_8(geom):
    g = geom
    x = wl.small_ints((g["N"], g["H"], g["W"], g["C"]), "f16", 95)
    w = wl.small_ints((g["R"], g["S"], g["C"], g["K"]), "f16", 96)
    P = (g["H"] + 2 * g["pad"][0] - g["R"]) // g["stride"][0] + 1
    Q = (g["W"] + 2 * g["pad"][1] - g["S"]) // g["stride"][1] + 1
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, g["stride"], g["pad"])
    ran = 0
    for krsc in (False, True):
        prob = al.problem(al.OP_CONV2D, g["N"] * P * Q, g["K"], g["R"] * g["S"] * g["C"], al.F16, al.F16,
                          conv_C=g["C"], transB=krsc)
        wt = w.permute(3, 0, 1, 2).contiguous() if krsc else w
        fn = al.alcop_conv2d_igemm_krsc if krsc else al.alcop_conv2d_igemm
        for n, s in enumerate(emu.space(prob)):
            if g["C"] % s.bk == 0:
                continue                                   # served by the one-tap gather, tested above
            y = torch.full((g["N"], P, Q, g["K"]), float("nan"), dtype=torch.float16)
            errs = emu.call(fn, x, wt, y, g["stride"], g["pad"], s, reads=[x, wt], writes=[y],
                            policy=emu.POLICIES[n % 4])
            assert not errs, (repr(s), krsc, errs[:4])
            assert _exact(y, ref), (repr(s), krsc)
            ran += 1
    assert ran >= 2


def test_conv_bias_relu_in_the_epilogue():
    x = wl.small_ints((2, 6, 5, 64), "f16", 97)
    w = wl.small_ints((3, 3, 64, 72), "f16", 98)
    bias = (torch.arange(72, dtype=torch.float32) % 9) - 4
    ref = oracle.epilogue(oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (1, 1), (1, 1)).reshape(-1, 72),
                          0.5, bias.double().numpy(), 1).reshape(2, 6, 5, 72)
    for krsc in (False, True):
        wt = w.permute(3, 0, 1, 2).contiguous() if krsc else w
        y = torch.full((2, 6, 5, 72), float("nan"), dtype=torch.float32)
        errs = emu.call(al.alcop_conv2d_igemm_fused, x, wt, y, (1, 1), (1, 1), 0.5, bias, 1, krsc,
                        al.sched(128, 64, 64, 64, 32, 3, 2, 1), reads=[x, wt, bias], writes=[y])
        assert not errs, errs[:4]
        assert _exact(y, ref), krsc


# ---- convolution with the input patch resident in LDS (schedule variant 1) ---------------------------
@pytest.mark.parametrize("geom", [
    dict(N=2, H=9, W=7, C=64, K=64, R=3, S=3, pad=(1, 1)),
    dict(N=1, H=20, W=18, C=64, K=72, R=3, S=3, pad=(1, 1)),      # several tiles per image
    dict(N=2, H=6, W=10, C=32, K=64, R=5, S=3, pad=(2, 0)),
    dict(N=1, H=8, W=8, C=64, K=64, R=1, S=1, pad=(0, 0)),
    dict(N=3, H=5, W=6, C=32, K=64, R=2, S=4, pad=(1, 2)),
])
def test_conv_patch_variant_exact_and_in_bounds(geom):
    g = geom
    dt = "f16"
    x = wl.small_ints((g["N"], g["H"], g["W"], g["C"]), dt, 101)
    w = wl.small_ints((g["R"], g["S"], g["C"], g["K"]), dt, 102)
    P = g["H"] + 2 * g["pad"][0] - g["R"] + 1
    Q = g["W"] + 2 * g["pad"][1] - g["S"] + 1
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (1, 1), g["pad"])
    prob = al.problem(al.OP_CONV2D, g["N"] * P * Q, g["K"], g["R"] * g["S"] * g["C"], al.F16, al.F16,
                      conv_C=g["C"])
    with emu._swapped():
        scheds = [s for s in al.alcop_sched_variants(prob) if s.variant == 1]
        assert scheds and all(al.alcop_sched_supported(prob, s) == al.OK for s in scheds)
        assert all(s.variant != 1 for s in al.alcop_sched_space(prob))
    for n, s in enumerate(scheds):
        for policy in (emu.POLICIES[n % 4], emu.POLICIES[(n + 2) % 4]):
            y = torch.full((g["N"], P, Q, g["K"]), float("nan"), dtype=torch.float16)
            errs = emu.call(al.alcop_conv2d_igemm, x, w, y, (1, 1), g["pad"], s,
                            reads=[x, w], writes=[y], policy=policy)
            assert not errs, (repr(s), policy, errs[:4])
            assert _exact(y, ref), (repr(s), policy)


def test_conv_patch_variant_is_refused_where_it_does_not_apply():
    x = wl.small_ints((1, 12, 12, 64), "f16", 103)
    w = wl.small_ints((3, 3, 64, 64), "f16", 104)
    s = al.sched(128, 64, 64, 64, 32, 2, 2, 0, variant=1)
    y = torch.zeros(1, 6, 6, 64, dtype=torch.float16)
    with pytest.raises(al.AlcopError) as e:                        # stride 2
        emu.call(al.alcop_conv2d_igemm, x, w, y, (2, 2), (1, 1), s, reads=[x, w], writes=[y])
    assert e.value.code == al.ERR_SCHED
    big = wl.small_ints((1, 4, 700, 64), "f16", 105)               # a halo of two 702-pixel rows: too much LDS
    yb = torch.zeros(1, 4, 700, 64, dtype=torch.float16)
    with pytest.raises(al.AlcopError) as e:
        emu.call(al.alcop_conv2d_igemm, big, w, yb, (1, 1), (1, 1), s, reads=[big, w], writes=[yb])
    assert e.value.code == al.ERR_SCHED
    with emu._swapped():
        gemm = al.problem(al.OP_GEMM, 128, 64, 64, al.F16, al.F16)
        assert al.alcop_sched_supported(gemm, al.sched(128, 64, 64, 64, 32, 2, 2, 0, variant=1)) == al.ERR_SCHED
        c32 = al.problem(al.OP_CONV2D, 144, 64, 9 * 32, al.F16, al.F16, conv_C=32)
        assert al.alcop_sched_supported(c32, s) == al.ERR_SCHED     # bk must equal the channel count


def test_conv_patch_variant_bf16_bias_relu_several_column_tiles():
    x = wl.small_ints((2, 7, 9, 64), "bf16", 111)
    w = wl.small_ints((3, 3, 64, 136), "bf16", 112)
    bias = (torch.arange(136, dtype=torch.float32) % 5) - 2
    ref = oracle.epilogue(oracle.conv2d(wl.bits(x), wl.bits(w), oracle.BF16, (1, 1), (1, 1)).reshape(-1, 136),
                          2.0, bias.double().numpy(), 1).reshape(2, 7, 9, 136)
    for raster in (1, 0):
        y = torch.full((2, 7, 9, 136), float("nan"), dtype=torch.float32)
        s = al.sched(128, 64, 64, 64, 32, 3, 2, 1, raster, 0, 1)
        errs = emu.call(al.alcop_conv2d_igemm_fused, x, w, y, (1, 1), (1, 1), 2.0, bias, 1, False, s,
                        reads=[x, w, bias], writes=[y], policy=(1, 1))
        assert not errs, errs[:4]
        assert _exact(y, ref), raster


def test_splitk_weight_gradient_layout_a_stored_k_by_m():
    # dW = X^T . dY: X is [tokens, in], dY is [tokens, out]; small output, long reduction axis
    tokens, fin, fout = 8 * 64 + 40, 136, 72
    X = wl.small_ints((tokens, fin), "f16", 121)
    dY = wl.small_ints((tokens, fout), "f16", 122)
    ref = oracle.gemm(wl.bits(X.t().contiguous()), wl.bits(dY), oracle.F16)
    for split in (3, 9):
        dW = torch.full((fin, fout), float("nan"), dtype=torch.float32)
        ws = _ws(1, fin, fout, split)
        errs = emu.call(al.alcop_gemm_splitk, X, dY, dW, split, ws, al.sched(128, 128, 64, 64, 64, 3, 2, 1),
                        transA=True, reads=[X, dY], writes=[dW, ws], policy=emu.POLICIES[split % 4])
        assert not errs, errs[:4]
        assert _exact(dW, ref), split


def test_k_tile_of_128_all_policies_and_l2_touches():
    for transB, s in ((0, al.sched(128, 128, 128, 64, 64, 2, 2, 1)), (1, al.sched(64, 64, 128, 32, 32, 3, 2, 1)),
                      (0, al.sched(64, 64, 128, 32, 32, 4, 2, 1, 1, 2))):
        for policy in emu.POLICIES:
            errs, ok = _gemm_case("f16", 0, transB, s, 2 * s.bm - 24, s.bn + 8, 5 * 128 + (0 if s.l2_prefetch else 40),
                                  policy, out="f32")
            assert not errs and ok, (repr(s), policy, errs[:4])


@pytest.mark.parametrize("geom", [
    dict(N=2, H=9, W=8, C=64, K=64, R=3, S=3, stride=(1, 1), pad=(2, 2), dil=(2, 2), krsc=False),
    dict(N=1, H=12, W=11, C=32, K=72, R=3, S=2, stride=(2, 1), pad=(3, 0), dil=(3, 2), krsc=False),
    dict(N=2, H=8, W=8, C=24, K=64, R=3, S=3, stride=(1, 1), pad=(2, 1), dil=(2, 1), krsc=True),
])
def test_dilated_convolution_exact_and_in_bounds(geom):
    g = geom
    x = wl.small_ints((g["N"], g["H"], g["W"], g["C"]), "f16", 131)
    w = wl.small_ints((g["R"], g["S"], g["C"], g["K"]), "f16", 132)
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, g["stride"], g["pad"], g["dil"])
    wk = w.permute(3, 0, 1, 2).contiguous() if g["krsc"] else w
    prob = al.problem(al.OP_CONV2D, ref.shape[0] * ref.shape[1] * ref.shape[2], g["K"],
                      g["R"] * g["S"] * g["C"], al.F16, al.F32, conv_C=g["C"], transB=g["krsc"])
    scheds = emu.space(prob)
    assert scheds
    for n, s in enumerate(scheds):
        y = torch.full(tuple(ref.shape), float("nan"), dtype=torch.float32)
        errs = emu.call(al.alcop_conv2d_igemm_dilated, x, wk, y, g["stride"], g["pad"], g["dil"],
                        krsc=g["krsc"], sched=s, reads=[x, wk], writes=[y], policy=emu.POLICIES[n % 4])
        assert not errs, (repr(s), errs[:4])
        assert _exact(y, ref), repr(s)
    # the patch kernels keep dilation 1
    if g["C"] == 64 and not g["krsc"]:
        y = torch.zeros(tuple(ref.shape), dtype=torch.float32)
        with pytest.raises(al.AlcopError) as e:
            emu.call(al.alcop_conv2d_igemm_dilated, x, wk, y, g["stride"], g["pad"], g["dil"],
                     sched=al.sched(256, 64, 64, 64, 64, 3, 2, 1, 1, 0, 1), reads=[x, wk], writes=[y])
        assert e.value.code == al.ERR_SCHED


# ---- persistent producer / consumer kernels (schedule variant 2) ---------------------------------
def _stream_scheds(prob):
    return [s for s in emu.space(prob, opt_in=True) if s.variant == 2]


@pytest.mark.parametrize("dt,transB", [("f16", 0), ("f16", 1), ("bf16", 0)])
def test_stream_kernels_batched_every_block_count(dt, transB, monkeypatch):
    # one block walks all tiles; two and three blocks interleave them; more blocks than tiles; one
    # k-tile per tile (the pipeline is all fill and drain), two with a partial one, five
    prob = al.problem(al.OP_BMM, 512, 512, 512, ADT[dt], ADT[dt], batch=3, transB=bool(transB))
    scheds = _stream_scheds(prob)
    assert scheds
    for n, s in enumerate(scheds):
        for blocks in (1, 2, 3, 1000):
            monkeypatch.setenv("ALCOP_STREAM_BLOCKS", str(blocks))
            for nk, extra in ((1, 0), (2, 8), (5, 0)):
                b, M, N, K = 2, 2 * s.bm + 24, s.bn + 8, nk * s.bk + extra
                A = wl.small_ints((b, M, K), dt, 500 + n)
                B = wl.small_ints((b, N, K) if transB else (b, K, N), dt, 501 + n)
                C = torch.full((b, M, N), float("nan"), dtype=torch.float32)
                policy = emu.POLICIES[(n + blocks + nk) % 4]
                errs = emu.call(al.alcop_bmm, A, B, C, s, transB=bool(transB), reads=[A, B], writes=[C],
                                policy=policy)
                ref = oracle.bmm(wl.bits(A), wl.bits(B), ODT[dt], transB=bool(transB))
                assert not errs, (repr(s), blocks, K, policy, errs[:4])
                assert _exact(C, ref), (repr(s), blocks, K, policy)


def test_stream_kernels_tile_list_dealt_by_xcd(monkeypatch):
    # 4 matrices of 2 x 2 tiles = 16 tiles and 8 blocks: the permuted tile list (one eighth of
    # the sequence per XCD) must still cover every tile exactly once; also 16 blocks and 24 tiles
    s = al.sched(64, 64, 64, 32, 32, 3, 2, 1, 1, 0, 2)
    for b, blocks in ((4, 8), (4, 16), (6, 8)):
        monkeypatch.setenv("ALCOP_STREAM_BLOCKS", str(blocks))
        A = wl.small_ints((b, 128, 136), "f16", 61)
        B = wl.small_ints((b, 128, 136), "f16", 62)
        C = torch.full((b, 128, 128), float("nan"), dtype=torch.float32)
        errs = emu.call(al.alcop_bmm, A, B, C, s, transB=True, reads=[A, B], writes=[C], policy=(1, 1))
        assert not errs, errs[:4]
        assert _exact(C, oracle.bmm(wl.bits(A), wl.bits(B), oracle.F16, transB=True)), (b, blocks)


def test_stream_kernels_convolution_gemm_and_fused_epilogue(monkeypatch):
    x = wl.small_ints((2, 9, 7, 64), "f16", 31)
    w = wl.small_ints((3, 3, 64, 64), "f16", 32)
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (1, 1), (1, 1))
    prob = al.problem(al.OP_CONV2D, 2 * 9 * 7, 64, 576, al.F16, al.F32, conv_C=64)
    scheds = _stream_scheds(prob)
    assert scheds
    for n, s in enumerate(scheds):
        for blocks in (1, 2, 1000):
            monkeypatch.setenv("ALCOP_STREAM_BLOCKS", str(blocks))
            y = torch.full((2, 9, 7, 64), float("nan"), dtype=torch.float32)
            errs = emu.call(al.alcop_conv2d_igemm, x, w, y, (1, 1), (1, 1), s, reads=[x, w], writes=[y],
                            policy=emu.POLICIES[(n + blocks) % 4])
            assert not errs, (repr(s), blocks, errs[:4])
            assert _exact(y, ref), (repr(s), blocks)
    # strided, dilated, ragged channel tile count per tap (C = 128, bk = 64: two k-tiles per tap)
    x = wl.small_ints((1, 11, 10, 128), "f16", 33)
    w = wl.small_ints((3, 2, 128, 72), "f16", 34)
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (2, 1), (2, 1), (2, 1))
    monkeypatch.setenv("ALCOP_STREAM_BLOCKS", "2")
    y = torch.full(tuple(ref.shape), float("nan"), dtype=torch.float32)
    errs = emu.call(al.alcop_conv2d_igemm_dilated, x, w, y, (2, 1), (2, 1), (2, 1),
                    sched=al.sched(128, 64, 64, 64, 32, 3, 2, 1, 1, 0, 2), reads=[x, w], writes=[y], policy=(1, 1))
    assert not errs, errs[:4]
    assert _exact(y, ref)
    # plain GEMM with bias and ReLU, fp16 output, three blocks over six tiles
    M, N, K = 3 * 128 - 8, 2 * 128 - 56, 3 * 64 + 16
    A = wl.small_ints((M, K), "f16", 35)
    B = wl.small_ints((K, N), "f16", 36)
    bias = torch.arange(N, dtype=torch.float32) - 90
    C = torch.full((M, N), float("nan"), dtype=torch.float16)
    monkeypatch.setenv("ALCOP_STREAM_BLOCKS", "3")
    errs = emu.call(al.alcop_gemm_fused, A, B, C, 0.5, bias, 1, al.sched(128, 128, 64, 64, 64, 3, 2, 1, 1, 0, 2),
                    reads=[A, B, bias], writes=[C], policy=(1, 0))
    assert not errs, errs[:4]
    ref = oracle.epilogue(oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16), 0.5, bias.double().numpy(), 1)
    assert _exact(C, ref)


@pytest.mark.parametrize("reg_stages", [2, 4])
def test_stream_kernel_planted_mistakes_are_noticed(reg_stages, monkeypatch):
    monkeypatch.setenv("ALCOP_STREAM_BLOCKS", "2")
    s = al.sched(128, 128, 64, 64, 64, 3, reg_stages, 1, 1, 0, 2)   # 4: the consumers' deep register pipeline
    b, M, N, K = 2, 256, 128, 5 * 64
    A = wl.small_ints((b, M, K), "f16", 1)
    B = wl.small_ints((b, K, N), "f16", 2)
    ref = oracle.bmm(wl.bits(A), wl.bits(B), oracle.F16)

    def run(policy, mutation):
        C = torch.full((b, M, N), float("nan"), dtype=torch.float32)
        errs = emu.call(al.alcop_bmm, A, B, C, s, reads=[A, B], writes=[C], policy=policy, mutation=mutation)
        return errs, _exact(C, ref)
    for policy in emu.POLICIES:
        errs, ok = run(policy, 0)
        assert not errs and ok
    assert not run((1, 0), 1)[1]          # a wait that lets too many loads stay in flight
    for policy in emu.POLICIES:
        assert not run(policy, 2)[1]      # no block barrier between producers and consumers
    assert not run((1, 0), 3)[1]          # producers do not wait for their loads
    errs, _ = run((1, 0), 4)              # consumers do not wait for their reads before the barrier
    assert errs and "may still be fetching" in " ".join(errs)


def test_stream_schedules_are_refused_where_they_do_not_apply():
    A = wl.small_ints((128, 64), "f16", 1)
    B = wl.small_ints((64, 128), "f16", 2)
    C = torch.zeros(128, 128, dtype=torch.float32)
    for bad in (al.sched(128, 128, 64, 64, 64, 3, 2, 1, 1, 4, 2),      # L2 touches
                al.sched(128, 128, 64, 64, 64, 3, 1, 0, 1, 0, 2),      # one register stage
                al.sched(128, 128, 64, 64, 64, 1, 2, 1, 1, 0, 2)):     # a ring of one slot
        with pytest.raises(al.AlcopError) as e:
            emu.call(al.alcop_gemm, A, B, C, bad, reads=[A, B], writes=[C])
        assert e.value.code == al.ERR_SCHED


# ---- tiles 192 wide: three 64-column LDS images per stage ------------------------------------
@pytest.mark.parametrize("dt,transA,transB", [("f16", 0, 0), ("bf16", 0, 0), ("f16", 1, 0), ("f16", 0, 1)])
def test_tiles_192_wide_exact_and_in_bounds(dt, transA, transB):
    prob = al.problem(al.OP_GEMM, 512, 768, 512, ADT[dt], ADT[dt], transB=bool(transB), transA=bool(transA))
    scheds = [s for s in emu.space(prob) if 192 in (s.bm, s.bn)]
    assert scheds
    for n, s in enumerate(scheds):
        # full tile; ragged in m and n (the last image partly, then wholly, beyond N); one k-tile,
        # several and a partial one; a second tile in each direction
        for M, N, K in ((s.bm, s.bn, s.bk), (s.bm - 24, s.bn - 40, 3 * s.bk + 8), (s.bm + 8, s.bn - 72, 5 * s.bk),
                        (s.bm + 40, 2 * s.bn - 8, 2 * s.bk + 16)):
            if transA:
                M = (M + 7) // 8 * 8
            for policy in (emu.POLICIES[n % 4], emu.POLICIES[(n + 2) % 4]):
                errs, ok = _gemm_case(dt, transA, transB, s, M, N, K, policy, out="f32" if n % 2 else dt, seed=40 + n)
                assert not errs, (repr(s), (M, N, K), policy, errs[:4])
                assert ok, (repr(s), (M, N, K), policy)


def test_tiles_192_wide_persistent_kernel_several_tiles_per_block(monkeypatch):
    prob = al.problem(al.OP_GEMM, 512, 768, 512, al.F16, al.F16)
    scheds = [s for s in emu.space(prob) if s.bn == 192 and s.variant == 2]
    assert scheds
    for s in scheds:
        for blocks in ("1", "2", "5"):
            monkeypatch.setenv("ALCOP_STREAM_BLOCKS", blocks)
            errs, ok = _gemm_case("f16", 0, 0, s, 2 * s.bm + 24, 3 * s.bn - 40, 3 * s.bk + 8, (1, 1), out="f32", seed=77)
            assert not errs, (repr(s), blocks, errs[:4])
            assert ok, (repr(s), blocks)


def test_tiles_192_wide_fused_epilogue_batched():
    b, M, N, K = 2, 300, 200, 104
    A = wl.small_ints((b, M, K), "f16", 4101)
    B = wl.small_ints((b, K, N), "f16", 4102)
    bias = (torch.arange(N, dtype=torch.float32) % 7) - 3
    ref = oracle.epilogue(oracle.bmm(wl.bits(A), wl.bits(B), oracle.F16), 0.5, bias.double().numpy(), 1)
    for s in (al.sched(256, 192, 32, 128, 96, 3, 2, 1), al.sched(256, 192, 64, 64, 96, 2, 2, 1)):
        C = torch.full((b, M, N), float("nan"), dtype=torch.float16)
        errs = emu.call(al.alcop_bmm_fused, A, B, C, 0.5, bias, 1, s, reads=[A, B, bias], writes=[C], policy=(1, 1))
        assert not errs, (repr(s), errs[:4])
        assert _exact(C, ref), repr(s)
