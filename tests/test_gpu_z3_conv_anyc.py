"""GPU parity of the convolution for channel counts that the k-tile does not divide (any multiple
of 8; every lane tracks the filter tap of its own chunk), RSCK and KRSC weights."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV, assert_close, feasible, to_f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("geom", [
    dict(N=2, H=30, W=28, C=8, K=64, R=7, S=7, stride=(2, 2), pad=(3, 3)),     # padded RGB stem
    dict(N=2, H=9, W=10, C=24, K=72, R=3, S=3, stride=(1, 1), pad=(1, 1)),
    dict(N=1, H=11, W=9, C=40, K=64, R=3, S=2, stride=(1, 2), pad=(0, 1)),
    dict(N=3, H=7, W=7, C=96, K=128, R=1, S=1, stride=(1, 1), pad=(0, 0)),
])
def test_integers_bit_exact_every_schedule(geom):
    g = geom
    x = wl.small_ints((g["N"], g["H"], g["W"], g["C"]), "f16", 811)
    w = wl.small_ints((g["R"], g["S"], g["C"], g["K"]), "f16", 812)
    P = (g["H"] + 2 * g["pad"][0] - g["R"]) // g["stride"][0] + 1
    Q = (g["W"] + 2 * g["pad"][1] - g["S"]) // g["stride"][1] + 1
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, g["stride"], g["pad"])
    xd = x.to(DEV)
    ran = 0
    for krsc in (False, True):
        prob = al.problem(al.OP_CONV2D, g["N"] * P * Q, g["K"], g["R"] * g["S"] * g["C"], al.F16, al.F32,
                          conv_C=g["C"], transB=krsc)
        wd = (w.permute(3, 0, 1, 2).contiguous() if krsc else w).to(DEV)
        fn = al.alcop_conv2d_igemm_krsc if krsc else al.alcop_conv2d_igemm
        for s in feasible(prob):
            if g["C"] % s.bk == 0:
                continue
            y = torch.full((g["N"], P, Q, g["K"]), float("nan"), dtype=torch.float32, device=DEV)
            fn(xd, wd, y, g["stride"], g["pad"], s)
            torch.cuda.synchronize()
            assert np.array_equal(to_f64(y), ref), (repr(s), krsc)
            ran += 1
    assert ran >= 6


def test_stem_layer_random_data_and_automatic_schedule():
    # 7x7 stride-2 convolution of a 3-channel image padded to 8 channels, 64 filters
    n, H, W, C, K = 4, 112, 112, 8, 64
    x = wl.normal((n, H, W, C), "f16", 821, scale=1.0)
    x[..., 3:] = 0
    w = wl.normal((7, 7, C, K), "f16", 822, scale=1.0 / np.sqrt(49 * 3))
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (2, 2), (3, 3))
    y = torch.full((n, 56, 56, K), float("nan"), dtype=torch.float16, device=DEV)
    al.alcop_conv2d_igemm(x.to(DEV), w.to(DEV), y, (2, 2), (3, 3), None)
    torch.cuda.synchronize()
    assert_close(to_f64(y), ref, "stem conv")
    assert np.max(np.abs(to_f64(y) - ref)) < 2e-2 * float(np.sqrt(np.mean(ref ** 2)))
