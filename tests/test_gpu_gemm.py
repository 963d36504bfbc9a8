"""GPU parity of alcop_gemm against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import ADT, DEV, ODT, TDT, assert_close, feasible, tile_key, to_f64

pytestmark = pytest.mark.gpu


def run_gemm(A, B, out, s, transB=False, poison=True):
    M = A.shape[0]
    N = B.shape[0] if transB else B.shape[1]
    C = torch.full((M, N), float("nan") if poison else 0.0, dtype=TDT[out], device=DEV)
    al.alcop_gemm(A.to(DEV), B.to(DEV), C, s, transB=transB)
    torch.cuda.synchronize()
    return C


@pytest.mark.parametrize("dt,transB", [("f16", False), ("bf16", False), ("f16", True), ("bf16", True)])
def test_small_integers_bit_exact_every_schedule(dt, transB):
    # 256^3, values in {-2..2}: every partial sum is an integer below 2^24, so fp32 accumulation
    # is exact in any order and the result must equal the oracle bit for bit, for every kernel.
    M = N = K = 256
    A = wl.small_ints((M, K), dt, 101)
    B = wl.small_ints((N, K) if transB else (K, N), dt, 102)
    ref = oracle.gemm(wl.bits(A), wl.bits(B), ODT[dt], transB=transB)
    prob = al.problem(al.OP_GEMM, M, N, K, ADT[dt], al.F32, transB=transB)
    scheds = feasible(prob)
    assert len(scheds) >= 12
    for s in scheds:
        got = to_f64(run_gemm(A, B, "f32", s, transB))
        assert np.array_equal(got, ref), repr(s)
    # fp16 output holds integers up to 2048 exactly (|sum| <= 4*256)
    if dt == "f16":
        for s in scheds[::7]:
            assert np.array_equal(to_f64(run_gemm(A, B, "f16", s, transB)), ref), repr(s)


def test_bf16_output_bit_exact_on_integers():
    # bf16 holds integers up to 256 exactly: K = 64 keeps |sum| <= 256
    A = wl.small_ints((256, 64), "bf16", 103)
    B = wl.small_ints((64, 256), "bf16", 104)
    ref = oracle.gemm(wl.bits(A), wl.bits(B), oracle.BF16)
    prob = al.problem(al.OP_GEMM, 256, 256, 64, al.BF16, al.BF16)
    for s in feasible(prob):
        assert np.array_equal(to_f64(run_gemm(A, B, "bf16", s)), ref), repr(s)


@pytest.mark.parametrize("dt,transB", [("f16", False), ("bf16", False), ("f16", True)])
def test_bit_identical_across_stage_counts(dt, transB):
    # pipelining must not change a single bit for a fixed tile / k-order (random data)
    M, N, K = 512, 384, 640
    A = wl.uniform((M, K), dt, 105)
    B = wl.uniform((N, K) if transB else (K, N), dt, 106)
    prob = al.problem(al.OP_GEMM, M, N, K, ADT[dt], al.F32, transB=transB)
    groups = {}
    for s in feasible(prob):
        groups.setdefault(tile_key(s), []).append(s)
    ref = oracle.gemm(wl.bits(A), wl.bits(B), ODT[dt], transB=transB)
    for key, ss in groups.items():
        base = run_gemm(A, B, "f32", ss[0], transB)
        assert_close(to_f64(base), ref, repr(ss[0]))
        for s in ss[1:]:
            other = run_gemm(A, B, "f32", s, transB)
            assert torch.equal(base.view(torch.int32), other.view(torch.int32)), (repr(ss[0]), repr(s))


def test_repeat_runs_are_deterministic():
    A = wl.uniform((512, 512), "f16", 107)
    B = wl.uniform((512, 512), "f16", 108)
    s = al.sched(128, 128, 64, 64, 64, 3, 2, 1)
    first = run_gemm(A, B, "f32", s)
    for _ in range(20):
        assert torch.equal(first.view(torch.int32), run_gemm(A, B, "f32", s).view(torch.int32))


def test_config_gemm256_random_and_integer():
    for name in ("gemm256", "gemm256_int"):
        cfg, A, B = wl.make_inputs(name)
        ref = oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16)
        got = to_f64(run_gemm(A, B, "f32", None))            # library picks the schedule
        if name.endswith("_int"):
            assert np.array_equal(got, ref)
        else:
            assert_close(got, ref, name)


def test_identity_and_permutation_exact():
    n = 256
    X = wl.uniform((n, n), "f16", 109)
    I = wl.identity(n, "f16")
    P, perm = wl.permutation(n, "f16", 110)
    Xv = to_f64(X)
    for s in [al.sched(128, 128, 64, 64, 64, 3, 2, 1), al.sched(64, 64, 32, 32, 32, 2, 1, 0),
              al.sched(256, 256, 32, 128, 128, 4, 2, 1)]:
        assert np.array_equal(to_f64(run_gemm(I, X, "f32", s)), Xv)
        assert np.array_equal(to_f64(run_gemm(X, I, "f32", s)), Xv)
        assert np.array_equal(to_f64(run_gemm(P, X, "f32", s)), Xv[perm])
        assert np.array_equal(to_f64(run_gemm(P, X, "f16", s)), Xv[perm])


@pytest.mark.parametrize("shape", [(200, 136, 192), (1, 8, 64), (129, 264, 128), (300, 72, 320), (64, 64, 64)])
@pytest.mark.parametrize("transB", [False, True])
def test_ragged_edges(shape, transB):
    # M not a multiple of the tile, N only a multiple of 8: zero-filled loads, masked stores
    M, N, K = shape
    A = wl.small_ints((M, K), "f16", 111)
    B = wl.small_ints((N, K) if transB else (K, N), "f16", 112)
    ref = oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16, transB=transB)
    for s in [al.sched(128, 128, 64, 64, 64, 3, 2, 1), al.sched(64, 64, 32, 32, 32, 2, 2, 1),
              al.sched(128, 128, 32, 64, 64, 1, 1, 0), al.sched(256, 256, 64, 128, 128, 2, 2, 1)]:
        assert np.array_equal(to_f64(run_gemm(A, B, "f32", s, transB)), ref), repr(s)


@pytest.mark.parametrize("K", [8, 40, 72, 96, 200, 328])
@pytest.mark.parametrize("transB", [False, True])
def test_partial_last_k_tile(K, transB):
    # K only a multiple of 8: the chunks of the last k-tile at k >= K are zero-filled
    M, N = 136, 72
    for dt in ("f16", "bf16"):
        A = wl.small_ints((M, K), dt, 117)
        B = wl.small_ints((N, K) if transB else (K, N), dt, 118)
        ref = oracle.gemm(wl.bits(A), wl.bits(B), ODT[dt], transB=transB)
        for s in [al.sched(128, 128, 64, 64, 64, 3, 2, 1), al.sched(64, 64, 32, 32, 32, 2, 2, 1),
                  al.sched(128, 128, 32, 64, 64, 1, 1, 0), al.sched(64, 64, 64, 32, 32, 2, 1, 0)]:
            assert np.array_equal(to_f64(run_gemm(A, B, "f32", s, transB)), ref), (dt, repr(s))


def test_masked_stores_do_not_touch_memory_outside_c():
    M, N, K = 100, 72, 128
    A = wl.small_ints((M, K), "f16", 113)
    B = wl.small_ints((K, N), "f16", 114)
    big = torch.full((M + 60, N + 56), -7.0, dtype=torch.float32, device=DEV)
    C = big[:M, :N]                                   # view: ldc = N + 56
    al.alcop_gemm(A.to(DEV), B.to(DEV), C, al.sched(128, 128, 64, 64, 64, 3, 2, 1))
    torch.cuda.synchronize()
    ref = oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16)
    assert np.array_equal(to_f64(C), ref)
    assert bool((big[M:, :] == -7.0).all()) and bool((big[:, N:] == -7.0).all())


def test_leading_dimensions_of_views():
    # operands that are column slices of larger matrices
    bigA = wl.uniform((256, 512), "f16", 115)
    bigB = wl.uniform((256, 640), "f16", 116)
    A = bigA[:, 128:384]
    B = bigB[:, 64:448]
    ref = oracle.gemm(wl.bits(A.contiguous()), wl.bits(B.contiguous()), oracle.F16)
    Ad, Bd = bigA.to(DEV)[:, 128:384], bigB.to(DEV)[:, 64:448]
    C = torch.empty(256, 384, dtype=torch.float32, device=DEV)
    al.alcop_gemm(Ad, Bd, C, al.sched(128, 128, 64, 64, 64, 2, 2, 1))
    torch.cuda.synchronize()
    assert_close(to_f64(C), ref, "views")


def test_infeasible_schedule_is_an_error_not_a_launch():
    A = torch.zeros(256, 256, dtype=torch.float16, device=DEV)
    C = torch.full((256, 256), 3.0, dtype=torch.float32, device=DEV)
    for bad in [al.sched(256, 256, 64, 128, 128, 4, 2, 1), al.sched(128, 128, 64, 64, 64, 1, 2, 1),
                al.sched(96, 96, 64, 32, 32, 2, 1, 0)]:
        with pytest.raises(al.AlcopError) as e:
            al.alcop_gemm(A, A, C, bad)
        assert e.value.code == al.ERR_SCHED
    torch.cuda.synchronize()
    assert bool((C == 3.0).all())


# ---- full-size configurations, in the launch configuration the benchmark times ------------------
def test_config_gemm2048_full_oracle_and_sweep():
    cfg, A, B = wl.make_inputs("gemm2048")
    ref = oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16)
    prob = al.problem(al.OP_GEMM, 2048, 2048, 2048, al.F16, al.F16)
    Ad, Bd = A.to(DEV), B.to(DEV)
    scheds = feasible(prob)
    # the sweep of the motivating example: every tile x k-tile x stage point that fits
    for s in scheds:
        C = torch.full((2048, 2048), float("nan"), dtype=torch.float16, device=DEV)
        al.alcop_gemm(Ad, Bd, C, s)
        torch.cuda.synchronize()
        assert_close(to_f64(C), ref, repr(s))


@pytest.mark.parametrize("name", ["ffn1", "ffn2"])
def test_config_transformer_linear_layers(name):
    cfg, A, B = wl.make_inputs(name)
    ref = oracle.gemm(wl.bits(A), wl.bits(B), oracle.BF16)
    for s in [None, al.sched(256, 256, 64, 128, 128, 2, 2, 1), al.sched(128, 128, 64, 64, 64, 3, 2, 1)]:
        got = to_f64(run_gemm(A, B, "bf16", s))
        assert_close(got, ref, name)


def test_config_gemm8192_sampled_rows():
    # 8192^3 is 5.5e11 multiply-adds: the oracle checks 256 seeded rows of C (all columns)
    cfg, A, B = wl.make_inputs("gemm8192")
    rows = np.sort(np.random.default_rng(8192).choice(8192, size=256, replace=False))
    ref = oracle.gemm(wl.bits(A[torch.from_numpy(rows)]), wl.bits(B), oracle.BF16)
    Ad, Bd = A.to(DEV), B.to(DEV)
    for s in [None, al.sched(256, 256, 64, 128, 128, 2, 2, 1), al.sched(256, 256, 32, 128, 64, 4, 2, 1)]:
        C = torch.full((8192, 8192), float("nan"), dtype=torch.bfloat16, device=DEV)
        al.alcop_gemm(Ad, Bd, C, s)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(C).all())
        assert_close(to_f64(C[torch.from_numpy(rows).to(DEV)]), ref, "gemm8192 " + repr(s))


def test_config_gemm4096_sampled_rows():
    # fp16 in and out, one 256 x 256 tile per compute unit: 512 seeded rows of C against the oracle
    cfg, A, B = wl.make_inputs("gemm4096")
    rows = np.sort(np.random.default_rng(4096).choice(4096, size=512, replace=False))
    ref = oracle.gemm(wl.bits(A[torch.from_numpy(rows)]), wl.bits(B), oracle.F16)
    Ad, Bd = A.to(DEV), B.to(DEV)
    for s in [None, al.sched(256, 256, 64, 128, 128, 2, 3, 1), al.sched(128, 128, 64, 64, 64, 3, 2, 0, 1, 0, 2)]:
        C = torch.full((4096, 4096), float("nan"), dtype=torch.float16, device=DEV)
        al.alcop_gemm(Ad, Bd, C, s)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(C).all())
        assert_close(to_f64(C[torch.from_numpy(rows).to(DEV)]), ref, "gemm4096 " + repr(s))
