"""Pins for the convolution oracle: a second route (explicit im2col matrix + the GEMM oracle),
the 1x1 case that is a plain GEMM, delta-tap weights (pin the direction of padding and the
absence of a kernel flip), tap counts at the border, brute force on a hand-sized case."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl


def _vals(t):
    return t.to(torch.float64).numpy()


def _im2col(xb, R, S, sh, sw, ph, pw):
    """uint16 matrix [N*P*Q, R*S*C]; out-of-image taps hold the pattern of +0.0."""
    N, H, W, C = xb.shape
    P = (H + 2 * ph - R) // sh + 1
    Q = (W + 2 * pw - S) // sw + 1
    out = np.zeros((N, P, Q, R, S, C), dtype=np.uint16)
    for p in range(P):
        for q in range(Q):
            for r in range(R):
                for s in range(S):
                    ih, iw = p * sh - ph + r, q * sw - pw + s
                    if 0 <= ih < H and 0 <= iw < W:
                        out[:, p, q, r, s, :] = xb[:, ih, iw, :]
    return out.reshape(N * P * Q, R * S * C), P, Q


@pytest.mark.parametrize("geom", [
    dict(N=2, H=6, W=5, C=4, K=3, R=3, S=3, sh=1, sw=1, ph=1, pw=1),
    dict(N=1, H=9, W=8, C=2, K=5, R=3, S=2, sh=2, sw=1, ph=0, pw=1),
    dict(N=3, H=7, W=7, C=8, K=8, R=1, S=1, sh=1, sw=1, ph=0, pw=0),
    dict(N=1, H=8, W=8, C=3, K=2, R=5, S=5, sh=1, sw=2, ph=2, pw=2),
])
def test_conv_equals_im2col_gemm(geom):
    g = geom
    x = wl.normal((g["N"], g["H"], g["W"], g["C"]), "f16", 31, 0.5)
    w = wl.normal((g["R"], g["S"], g["C"], g["K"]), "f16", 32, 0.5)
    got = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (g["sh"], g["sw"]), (g["ph"], g["pw"]))
    col, P, Q = _im2col(wl.bits(x), g["R"], g["S"], g["sh"], g["sw"], g["ph"], g["pw"])
    wm = wl.bits(w).reshape(g["R"] * g["S"] * g["C"], g["K"])
    want = oracle.gemm(col, wm, oracle.F16).reshape(g["N"], P, Q, g["K"])
    # zero taps add +0.0 in the GEMM route and are skipped in the direct one: same fp64 bits
    assert got.shape == want.shape
    assert np.array_equal(got, want)


def test_one_by_one_is_a_gemm():
    N, H, W, C, K = 2, 5, 4, 16, 12
    x = wl.normal((N, H, W, C), "bf16", 33, 0.5)
    w = wl.normal((1, 1, C, K), "bf16", 34, 0.5)
    got = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.BF16)
    want = oracle.gemm(wl.bits(x).reshape(N * H * W, C), wl.bits(w).reshape(C, K), oracle.BF16)
    assert np.array_equal(got.reshape(N * H * W, K), want)


def test_brute_force_hand_sized():
    N, H, W, C, K = 1, 4, 4, 2, 2
    x = wl.small_ints((N, H, W, C), "f16", 35)
    w = wl.small_ints((3, 3, C, K), "f16", 36)
    got = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (1, 1), (1, 1))
    xv, wv = _vals(x), _vals(w)
    want = np.zeros((N, 4, 4, K))
    for p in range(4):
        for q in range(4):
            for k in range(K):
                s = 0.0
                for r in range(3):
                    for ss in range(3):
                        for c in range(C):
                            ih, iw = p - 1 + r, q - 1 + ss
                            if 0 <= ih < H and 0 <= iw < W:
                                s += xv[0, ih, iw, c] * wv[r, ss, c, k]
                want[0, p, q, k] = s
    assert np.array_equal(got, want)


def test_delta_taps_pin_shift_direction():
    N, H, W, C = 2, 6, 7, 4
    x = wl.normal((N, H, W, C), "f16", 37, 1.0)
    xv = _vals(x)
    for (r0, s0) in [(1, 1), (0, 1), (2, 1), (1, 0), (1, 2), (0, 0), (2, 2)]:
        w = torch.zeros(3, 3, C, C, dtype=torch.float16)
        for c in range(C):
            w[r0, s0, c, c] = 1.0
        got = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (1, 1), (1, 1))
        # y[n,p,q,c] = x[n, p-1+r0, q-1+s0, c], zero outside
        want = np.zeros_like(xv)
        for p in range(H):
            for q in range(W):
                ih, iw = p - 1 + r0, q - 1 + s0
                if 0 <= ih < H and 0 <= iw < W:
                    want[:, p, q, :] = xv[:, ih, iw, :]
        assert np.array_equal(got, want), (r0, s0)


def test_all_ones_counts_in_bounds_taps():
    N, H, W, C, K = 1, 5, 6, 3, 2
    x = np.full((N, H, W, C), 0x3C00, dtype=np.uint16)
    w = np.full((3, 3, C, K), 0x3C00, dtype=np.uint16)
    got = oracle.conv2d(x, w, oracle.F16, (1, 1), (1, 1))
    assert got[0, 2, 2, 0] == 9 * C          # interior
    assert got[0, 0, 2, 1] == 6 * C          # edge
    assert got[0, 2, 0, 0] == 6 * C
    assert got[0, 0, 0, 0] == 4 * C          # corners
    assert got[0, H - 1, W - 1, 1] == 4 * C
    assert got.sum() == K * C * sum(
        sum(1 for r in range(3) for s in range(3) if 0 <= p - 1 + r < H and 0 <= q - 1 + s < W)
        for p in range(H) for q in range(W))


def test_matches_torch_conv2d_on_integers():
    # a library convolution on inputs where it is exact (small integers, fp64)
    N, H, W, C, K = 2, 9, 10, 6, 5
    x = wl.small_ints((N, H, W, C), "f16", 38)
    w = wl.small_ints((3, 3, C, K), "f16", 39)
    for stride, pad in [((1, 1), (1, 1)), ((2, 2), (1, 1)), ((1, 2), (0, 1))]:
        got = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, stride, pad)
        ref = torch.nn.functional.conv2d(
            x.to(torch.float64).permute(0, 3, 1, 2), w.to(torch.float64).permute(3, 2, 0, 1),
            stride=stride, padding=pad).permute(0, 2, 3, 1).numpy()
        assert np.array_equal(got, ref)


# ---- dilation (not in the paper; the dilated routine is pinned on its own) -----------------------
@pytest.mark.parametrize("geom", [
    dict(N=2, H=9, W=8, C=3, K=4, R=3, S=3, stride=(1, 1), pad=(2, 2), dil=(2, 2)),
    dict(N=1, H=11, W=10, C=2, K=3, R=3, S=2, stride=(2, 1), pad=(3, 0), dil=(3, 2)),
    dict(N=2, H=7, W=7, C=4, K=2, R=2, S=3, stride=(1, 2), pad=(0, 1), dil=(1, 2)),
])
def test_dilated_conv_against_a_library_convolution_on_integers(geom):
    g = geom
    x = wl.small_ints((g["N"], g["H"], g["W"], g["C"]), "f16", 41)
    w = wl.small_ints((g["R"], g["S"], g["C"], g["K"]), "f16", 42)
    got = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, g["stride"], g["pad"], g["dil"])
    want = torch.nn.functional.conv2d(x.double().permute(0, 3, 1, 2), w.double().permute(3, 2, 0, 1),
                                      stride=g["stride"], padding=g["pad"], dilation=g["dil"])
    assert np.array_equal(got, want.permute(0, 2, 3, 1).numpy())


def test_dilated_routine_with_dilation_one_is_the_plain_routine():
    import ctypes
    x = wl.normal((2, 6, 7, 5), "bf16", 43, 0.5)
    w = wl.normal((3, 2, 5, 4), "bf16", 44, 0.5)
    plain = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.BF16, (2, 1), (1, 1))
    xb, wb = np.ascontiguousarray(wl.bits(x)), np.ascontiguousarray(wl.bits(w))
    y = np.empty_like(plain)
    rc = oracle._load().alcop_oracle_conv2d_dilated(oracle._p16(xb), oracle._p16(wb), oracle._p64(y),
                                                   2, 6, 7, 5, 4, 3, 2, 2, 1, 1, 1, 1, 1, oracle.BF16)
    assert rc == 0 and np.array_equal(y, plain)


def test_dilated_delta_taps_shift_by_the_dilation():
    # one nonzero tap (r0, s0) with identity channels: y[p, q] = x[p - pad + r0*dh, q - pad + s0*dw]
    N, H, W, C = 1, 8, 9, 4
    x = wl.normal((N, H, W, C), "f16", 45, 1.0)
    xv = _vals(x)
    dh, dw, ph, pw = 2, 3, 2, 3
    for (r0, s0) in [(0, 0), (1, 1), (2, 0), (0, 2), (2, 2)]:
        w = torch.zeros(3, 3, C, C, dtype=torch.float16)
        w[r0, s0] = torch.eye(C, dtype=torch.float16)
        got = oracle.conv2d(wl.bits(x), wl.bits(w), oracle.F16, (1, 1), (ph, pw), (dh, dw))
        assert got.shape == (N, H, W, C)          # "same" padding for a 3x3 filter: pad = dilation
        want = np.zeros_like(got)
        for p in range(H):
            for q in range(W):
                ih, iw = p - ph + r0 * dh, q - pw + s0 * dw
                if 0 <= ih < H and 0 <= iw < W:
                    want[:, p, q, :] = xv[:, ih, iw, :]
        assert np.array_equal(got, want), (r0, s0)
