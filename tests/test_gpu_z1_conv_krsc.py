"""GPU parity of alcop_conv2d_igemm_krsc (weights stored [K][R][S][C]) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV, ODT, TDT, assert_close, feasible, to_f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("geom", [
    dict(N=2, H=12, W=10, C=64, K=72, R=3, S=3, stride=(1, 1), pad=(1, 1)),
    dict(N=3, H=9, W=9, C=32, K=64, R=3, S=2, stride=(2, 1), pad=(1, 0)),
])
def test_integers_bit_exact_every_schedule(geom):
    g = geom
    x = wl.small_ints((g["N"], g["H"], g["W"], g["C"]), "f16", 801)
    w = wl.small_ints((g["R"], g["S"], g["C"], g["K"]), "f16", 802)
    wk = w.permute(3, 0, 1, 2).contiguous()
    P = (g["H"] + 2 * g["pad"][0] - g["R"]) // g["stride"][0] + 1
    Q = (g["W"] + 2 * g["pad"][1] - g["S"]) // g["stride"][1] + 1
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, g["stride"], g["pad"])
    prob = al.problem(al.OP_CONV2D, g["N"] * P * Q, g["K"], g["R"] * g["S"] * g["C"], al.F16, al.F32,
                      conv_C=g["C"], transB=True)
    scheds = [s for s in feasible(prob) if g["C"] % s.bk == 0]     # one filter tap per k-tile
    assert scheds
    xd, wd = x.to(DEV), wk.to(DEV)
    for s in scheds:
        y = torch.full((g["N"], P, Q, g["K"]), float("nan"), dtype=torch.float32, device=DEV)
        al.alcop_conv2d_igemm_krsc(xd, wd, y, g["stride"], g["pad"], s)
        torch.cuda.synchronize()
        assert np.array_equal(to_f64(y), ref), repr(s)


def test_config_conv14_equals_the_rsck_result_within_tolerance():
    cfg, x, w = wl.make_inputs("conv14")
    ref = oracle.conv2d(wl.bits(x), wl.bits(w), ODT[cfg["dtype"]], (1, 1), (1, 1))
    n, H, W, K = cfg["N"], cfg["H"], cfg["W"], cfg["K"]
    y = torch.full((n, H, W, K), float("nan"), dtype=TDT[cfg["out"]], device=DEV)
    al.alcop_conv2d_igemm_krsc(x.to(DEV), w.permute(3, 0, 1, 2).contiguous().to(DEV), y, (1, 1), (1, 1), None)
    torch.cuda.synchronize()
    assert_close(to_f64(y), ref, "conv14 KRSC")
    scale = float(np.sqrt(np.mean(ref ** 2)))
    assert np.max(np.abs(to_f64(y) - ref)) < 2e-2 * scale


def test_conv_bias_relu_in_the_epilogue():
    x = wl.small_ints((2, 12, 10, 64), "f16", 831)
    w = wl.small_ints((3, 3, 64, 72), "f16", 832)
    bias = (torch.arange(72, dtype=torch.float32) % 9) - 4
    ref = oracle.epilogue(oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (1, 1), (1, 1)).reshape(-1, 72),
                          0.5, bias.double().numpy(), 1).reshape(2, 12, 10, 72)
    for krsc in (False, True):
        wt = (w.permute(3, 0, 1, 2).contiguous() if krsc else w).to(DEV)
        y = torch.full((2, 12, 10, 72), float("nan"), dtype=torch.float32, device=DEV)
        al.alcop_conv2d_igemm_fused(x.to(DEV), wt, y, (1, 1), (1, 1), 0.5, bias.to(DEV), 1, krsc,
                                    al.sched(128, 64, 64, 64, 32, 3, 2, 1))
        torch.cuda.synchronize()
        assert np.array_equal(to_f64(y), ref), krsc
