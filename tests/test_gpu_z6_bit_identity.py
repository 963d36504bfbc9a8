"""Same bits for every pipelining variant of a tile, on random data, for the operators beyond the
plain GEMM: convolution with each of its three gathers (one tap per k-tile, per-lane taps for any
channel count, input patch resident in LDS), both weight layouts, and the batched products.  The
order of the matrix instructions per accumulator does not depend on stages, register stages or
fusion, so a difference in a single bit means that a ring slot was read before it had landed or
refilled before it had been read.  One variant per tile is also compared with the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV, assert_close, to_f64

pytestmark = pytest.mark.gpu


def _groups(prob, keep=lambda s: True, variants=False):
    found = al.alcop_sched_space(prob) + (al.alcop_sched_variants(prob) if variants else [])
    by_tile = {}
    for s in found:
        if s.l2_prefetch == 0 and al.alcop_sched_supported(prob, s) == al.OK and keep(s):
            # the persistent kernels (variant 2) accumulate in the same order as the default ones
            by_tile.setdefault((s.bm, s.bn, s.bk, s.wm, s.wn, 1 if s.variant == 1 else 0), []).append(s)
    return by_tile


def _same_bits(outs, what):
    first = outs[0][1].view(torch.int16)
    for s, y in outs[1:]:
        assert torch.equal(y.view(torch.int16), first), "%s: %r differs from %r" % (what, s, outs[0][0])


@pytest.mark.parametrize("C,krsc", [(64, False), (64, True), (40, False), (24, True)])
def test_convolution_every_gather_and_weight_layout(C, krsc):
    # 3 x 3, 2 images of 19 x 17: 646 rows (a ragged last tile for every tile height), K = 72
    # (ragged), 9 C deep: 9 k-tiles of 64 for C = 64, a partial last k-tile for C = 40 and 24
    N, H, W, K = 2, 19, 17, 72
    x = wl.normal((N, H, W, C), "f16", 1300 + C, 1.0)
    w = wl.normal((3, 3, C, K), "f16", 1301 + C, 1.0 / (9 * C) ** 0.5)
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (1, 1), (1, 1))
    wd = (w.permute(3, 0, 1, 2).contiguous() if krsc else w).to(DEV)
    xd = x.to(DEV)
    prob = al.problem(al.OP_CONV2D, N * H * W, K, 9 * C, al.F16, al.F16, conv_C=C, transB=krsc)
    groups = _groups(prob, variants=not krsc)
    assert groups
    seen_variant = False
    for tile, scheds in groups.items():
        outs = []
        for s in scheds:
            y = torch.full((N, H, W, K), float("nan"), dtype=torch.float16, device=DEV)
            try:
                if krsc:
                    al.alcop_conv2d_igemm_krsc(xd, wd, y, (1, 1), (1, 1), s)
                else:
                    al.alcop_conv2d_igemm(xd, wd, y, (1, 1), (1, 1), s)
            except al.AlcopError as e:
                # whether a patch kernel can serve a call depends on the image size (its patch
                # must fit the LDS): such a schedule is refused, not run
                assert s.variant == 1 and e.code == al.ERR_SCHED, repr(s)
                continue
            outs.append((s, y))
        torch.cuda.synchronize()
        if not outs:
            continue
        assert_close(to_f64(outs[0][1]), ref, repr(outs[0][0]))
        _same_bits(outs, "conv C=%d krsc=%d tile %r" % (C, krsc, tile))
        seen_variant = seen_variant or tile[5] == 1
    if C == 64 and not krsc:
        assert seen_variant          # the LDS-resident patch kernels took part


def test_strided_convolution():
    N, H, W, C, K = 3, 15, 14, 64, 64
    x = wl.normal((N, H, W, C), "f16", 1310, 1.0)
    w = wl.normal((3, 3, C, K), "f16", 1311, 1.0 / (9 * C) ** 0.5)
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (2, 2), (1, 1))
    P, Q = (H + 2 - 3) // 2 + 1, (W + 2 - 3) // 2 + 1
    prob = al.problem(al.OP_CONV2D, N * P * Q, K, 9 * C, al.F16, al.F16, conv_C=C)
    xd, wd = x.to(DEV), w.to(DEV)
    for tile, scheds in _groups(prob).items():
        outs = []
        for s in scheds:
            y = torch.full((N, P, Q, K), float("nan"), dtype=torch.float16, device=DEV)
            al.alcop_conv2d_igemm(xd, wd, y, (2, 2), (1, 1), s)
            outs.append((s, y))
        torch.cuda.synchronize()
        assert_close(to_f64(outs[0][1]), ref, repr(outs[0][0]))
        _same_bits(outs, "strided conv tile %r" % (tile,))


@pytest.mark.parametrize("transB,shape", [(True, (5, 200, 264, 64)), (False, (5, 136, 64, 520)),
                                          (True, (3, 264, 136, 328))])
def test_batched_products(transB, shape):
    # attention-shaped: a short reduction axis (one k-tile of 64: the pipeline never fills), a
    # long one, and a ragged one; ragged M and N
    b, M, N, K = shape
    A = wl.normal((b, M, K), "f16", 1320, 0.5)
    B = wl.normal((b, N, K) if transB else (b, K, N), "f16", 1321, 0.5)
    ref = oracle.bmm(wl.bits(A), wl.bits(B), oracle.F16, transB=transB)
    prob = al.problem(al.OP_BMM, M, N, K, al.F16, al.F16, batch=b, transB=transB)
    Ad, Bd = A.to(DEV), B.to(DEV)
    groups = _groups(prob)
    assert groups
    for tile, scheds in groups.items():
        outs = []
        for s in scheds:
            Cd = torch.full((b, M, N), float("nan"), dtype=torch.float16, device=DEV)
            al.alcop_bmm(Ad, Bd, Cd, s, transB=transB)
            outs.append((s, Cd))
        torch.cuda.synchronize()
        assert_close(to_f64(outs[0][1]), ref, repr(outs[0][0]))
        _same_bits(outs, "bmm transB=%d tile %r" % (transB, tile))


def test_lds_swizzle_is_a_pure_permutation_same_bits_without_it():
    # the measurement library's no-swizzle variant leaves the LDS tile images unpermuted; loader and
    # reader agree on any permutation, so the product must come out bit for bit the same
    from paper_2210_16691_amd import diag
    names = diag.configs()
    for want, dt in (("f16 128x128x64 w64x64 S4 R2 F1", "f16"), ("bf16 256x256x32 w128x64 S3 R2 F1", "bf16")):
        i = names.index(want)
        A = wl.uniform((512, 256), dt, 9101).to(DEV)
        B = wl.uniform((256, 512), dt, 9102).to(DEV)
        C0 = torch.full((512, 512), float("nan"), dtype=A.dtype, device=DEV)
        C1 = torch.full((512, 512), float("nan"), dtype=A.dtype, device=DEV)
        diag.alcop_diag_time(i, diag.FULL, A, B, C0, 2)
        diag.alcop_diag_time(i, diag.NO_SWIZZLE, A, B, C1, 2)
        torch.cuda.synchronize()
        assert torch.equal(C0.view(torch.int16), C1.view(torch.int16)), want
        ref = oracle.gemm(wl.bits(A.cpu()), wl.bits(B.cpu()), oracle.F16 if dt == "f16" else oracle.BF16)
        assert_close(to_f64(C1), ref, want)
