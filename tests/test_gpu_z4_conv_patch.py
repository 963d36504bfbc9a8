"""GPU parity of the convolution variant that keeps the input patch of a tile in LDS (schedule
variant 1: stride 1, channel count equal to the k-tile, RSCK weights) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV, ODT, TDT, assert_close, to_f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("geom", [
    dict(N=2, H=12, W=10, C=64, K=72, R=3, S=3, pad=(1, 1)),
    dict(N=1, H=30, W=34, C=64, K=64, R=3, S=3, pad=(1, 1)),      # several tiles per image
    dict(N=2, H=9, W=13, C=32, K=64, R=5, S=3, pad=(2, 0)),
    dict(N=3, H=8, W=8, C=64, K=128, R=1, S=1, pad=(0, 0)),
])
def test_integers_bit_exact_every_variant_schedule(geom):
    g = geom
    x = wl.small_ints((g["N"], g["H"], g["W"], g["C"]), "f16", 841)
    w = wl.small_ints((g["R"], g["S"], g["C"], g["K"]), "f16", 842)
    P = g["H"] + 2 * g["pad"][0] - g["R"] + 1
    Q = g["W"] + 2 * g["pad"][1] - g["S"] + 1
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (1, 1), g["pad"])
    prob = al.problem(al.OP_CONV2D, g["N"] * P * Q, g["K"], g["R"] * g["S"] * g["C"], al.F16, al.F32,
                      conv_C=g["C"])
    scheds = al.alcop_sched_variants(prob)
    assert len(scheds) >= 6
    xd, wd = x.to(DEV), w.to(DEV)
    for s in scheds:
        y = torch.full((g["N"], P, Q, g["K"]), float("nan"), dtype=torch.float32, device=DEV)
        al.alcop_conv2d_igemm(xd, wd, y, (1, 1), g["pad"], s)
        torch.cuda.synchronize()
        assert np.array_equal(to_f64(y), ref), repr(s)


def test_config_conv56_with_the_patch_variant_and_in_the_tuner():
    cfg, x, w = wl.make_inputs("conv56")
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), ODT[cfg["dtype"]], (1, 1), (1, 1))
    n, H, W, C, K = cfg["N"], cfg["H"], cfg["W"], cfg["C"], cfg["K"]
    xd, wd = x.to(DEV), w.to(DEV)
    y = torch.full((n, H, W, K), float("nan"), dtype=TDT[cfg["out"]], device=DEV)
    al.alcop_conv2d_igemm(xd, wd, y, (1, 1), (1, 1), al.sched(256, 64, 64, 64, 64, 3, 2, 1, variant=1))
    torch.cuda.synchronize()
    assert_close(to_f64(y), ref, "conv56 patch variant")
    assert np.max(np.abs(to_f64(y) - ref)) < 2e-2 * float(np.sqrt(np.mean(ref ** 2)))
    # the tuner prunes nothing here (stride 1, the patch fits) and times variants when asked to
    prob = al.problem(al.OP_CONV2D, n * H * W, K, 9 * C, al.F16, al.F16, conv_C=C)
    conv = (n, H, W, C, K, 3, 3, 1, 1, 1, 1)
    plain = al.alcop_tune(prob, xd, wd, y, top_k=0, model=0, iters=3, conv=conv)
    both = al.alcop_tune(prob, xd, wd, y, top_k=0, model=0, iters=3, conv=conv, variants=True)
    assert both.space == plain.space + len(al.alcop_sched_variants(prob))
    assert all(s.variant != 1 for s, _, _ in plain.log)
    assert any(s.variant == 1 for s, _, _ in both.log)
    # stride 2: every patch variant is pruned
    x2 = wl.small_ints((2, 16, 16, 64), "f16", 843).to(DEV)
    y2 = torch.empty(2, 8, 8, 64, dtype=torch.float16, device=DEV)
    p2 = al.problem(al.OP_CONV2D, 2 * 8 * 8, 64, 9 * 64, al.F16, al.F16, conv_C=64)
    c2 = (2, 16, 16, 64, 64, 3, 3, 2, 2, 1, 1)
    a = al.alcop_tune(p2, x2, wd, y2, top_k=0, model=0, iters=2, conv=c2)
    b = al.alcop_tune(p2, x2, wd, y2, top_k=0, model=0, iters=2, conv=c2, variants=True)
    # (the opt-in kernels that are not patch convolutions stay: k-tile 128, deep persistent consumers)
    others = [s for s in al.alcop_sched_variants(p2) if s.variant != 1]
    assert b.space == a.space + len(others)
    assert not any(s.variant == 1 for s, _, _ in b.log)
    with pytest.raises(al.AlcopError) as e:
        al.alcop_conv2d_igemm(x2, wd, y2, (2, 2), (1, 1), al.sched(128, 64, 64, 64, 32, 2, 2, 1, variant=1))
    assert e.value.code == al.ERR_SCHED
