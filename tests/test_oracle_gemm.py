"""Pins for the GEMM / BMM oracle against things other than itself: brute-force Python loops,
identity / permutation operands, closed forms, exact integer arithmetic, a library matmul on
inputs where that matmul is exact.  Each is chosen so that a plausible mistake (transposed
operand, wrong leading dimension, dropped term, wrong batch stride) fails at least one."""
import numpy as np
import pytest

import oracle
import workloads as wl

DT = {"f16": oracle.F16, "bf16": oracle.BF16}


def _vals(t):
    return t.to(dtype=__import__("torch").float64).numpy()


def _brute(Av, Bv):
    M, K = Av.shape
    N = Bv.shape[1]
    C = np.zeros((M, N))
    for i in range(M):
        for j in range(N):
            s = 0.0
            for k in range(K):
                s += float(Av[i, k]) * float(Bv[k, j])
            C[i, j] = s
    return C


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 7), (8, 8, 8), (5, 2, 9)])
def test_brute_force_tiny(dt, shape):
    M, N, K = shape
    A = wl.uniform((M, K), dt, 1)
    B = wl.uniform((K, N), dt, 2)
    got = oracle.gemm(wl.bits(A), wl.bits(B), DT[dt])
    assert np.array_equal(got, _brute(_vals(A), _vals(B)))     # same k order -> same bits


@pytest.mark.parametrize("tA", [False, True])
@pytest.mark.parametrize("tB", [False, True])
def test_transposed_storage(tA, tB):
    M, N, K = 6, 10, 14
    A = wl.uniform((M, K), "f16", 3)
    B = wl.uniform((K, N), "f16", 4)
    want = _brute(_vals(A), _vals(B))
    Ab = wl.bits(A.t().contiguous()) if tA else wl.bits(A)
    Bb = wl.bits(B.t().contiguous()) if tB else wl.bits(B)
    got = oracle.gemm(Ab, Bb, oracle.F16, transA=tA, transB=tB)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_identity_and_permutation(dt):
    n, m = 48, 20
    X = wl.uniform((n, m), dt, 5)
    Y = wl.uniform((m, n), dt, 6)
    I = wl.identity(n, dt)
    P, perm = wl.permutation(n, dt, 7)
    Xv, Yv = _vals(X), _vals(Y)
    assert np.array_equal(oracle.gemm(wl.bits(I), wl.bits(X), DT[dt]), Xv)          # I.X = X
    assert np.array_equal(oracle.gemm(wl.bits(Y), wl.bits(I), DT[dt]), Yv)          # Y.I = Y
    assert np.array_equal(oracle.gemm(wl.bits(P), wl.bits(X), DT[dt]), Xv[perm])    # rows permuted
    # (Y.P)[i, perm[k]] = Y[i, k]
    got = oracle.gemm(wl.bits(Y), wl.bits(P), DT[dt])
    want = np.empty_like(Yv)
    want[:, perm] = Yv
    assert np.array_equal(got, want)


def test_all_ones_and_rank_one():
    M, N, K = 9, 13, 37
    ones = np.full((M, K), 0x3C00, dtype=np.uint16)
    onesB = np.full((K, N), 0x3C00, dtype=np.uint16)
    assert np.array_equal(oracle.gemm(ones, onesB, oracle.F16), np.full((M, N), float(K)))
    u = wl.small_ints((M, 1), "f16", 8, -3, 3)
    v = wl.small_ints((1, N), "f16", 9, -3, 3)
    A = u.expand(M, K).contiguous()
    B = v.expand(K, N).contiguous()
    want = K * _vals(u) * _vals(v)
    assert np.array_equal(oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16), want)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_small_integers_exact_vs_int64_and_library(dt):
    M, N, K = 70, 50, 300
    A = wl.small_ints((M, K), dt, 10)
    B = wl.small_ints((K, N), dt, 11)
    got = oracle.gemm(wl.bits(A), wl.bits(B), DT[dt])
    Ai = _vals(A).astype(np.int64)
    Bi = _vals(B).astype(np.int64)
    assert np.array_equal(got, (Ai @ Bi).astype(np.float64))          # exact integer arithmetic
    assert np.array_equal(got, _vals(A) @ _vals(B))                  # fp64 library matmul is exact here


def test_linearity_on_integers():
    M, N, K = 12, 16, 40
    A = wl.small_ints((M, K), "f16", 12)
    B1 = wl.small_ints((K, N), "f16", 13)
    B2 = wl.small_ints((K, N), "f16", 14)
    B12 = (B1.float() + B2.float()).half()
    f = lambda B: oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16)
    assert np.array_equal(f(B12), f(B1) + f(B2))


def test_random_close_to_library_matmul():
    # on non-integer data the library matmul sums in another order: agreement to fp64 rounding
    M, N, K = 64, 96, 512
    A = wl.uniform((M, K), "f16", 15)
    B = wl.uniform((K, N), "f16", 16)
    got = oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16)
    want = _vals(A) @ _vals(B)
    assert np.max(np.abs(got - want)) < 1e-11


def test_leading_dimension_is_respected():
    # a sub-matrix view: the oracle must honour the shapes it is given, not a stale stride
    A = wl.uniform((10, 24), "f16", 17)
    B = wl.uniform((24, 6), "f16", 18)
    full = oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16)
    part = oracle.gemm(wl.bits(A[:, :16].contiguous()), wl.bits(B[:16].contiguous()), oracle.F16)
    assert np.array_equal(part, _brute(_vals(A[:, :16]), _vals(B[:16])))
    assert not np.array_equal(part, full)


# ---- batched -------------------------------------------------------------------------------
def test_bmm_equals_gemm_per_batch():
    b, M, N, K = 5, 12, 20, 28
    A = wl.normal((b, M, K), "f16", 19, 0.125)
    B = wl.normal((b, K, N), "f16", 20, 0.125)
    got = oracle.bmm(wl.bits(A), wl.bits(B), oracle.F16)
    for i in range(b):
        assert np.array_equal(got[i], oracle.gemm(wl.bits(A[i]), wl.bits(B[i]), oracle.F16))
        assert np.array_equal(got[i], _brute(_vals(A[i]), _vals(B[i])))


def test_bmm_qkt_symmetric_and_matches_brute():
    b, L, d = 3, 10, 6
    Q = wl.normal((b, L, d), "f16", 21, 0.125)
    got = oracle.bmm(wl.bits(Q), wl.bits(Q), oracle.F16, transB=True)        # Q.Q^T
    for i in range(b):
        assert np.array_equal(got[i], got[i].T)
        assert np.array_equal(got[i], _brute(_vals(Q[i]), _vals(Q[i]).T))


def test_bmm_pv_row_sums_and_one_hot_gather():
    b, L, d = 2, 24, 8
    P = wl.softmax_rows((b, L, L), "f16", 22)
    ones = np.full((b, L, d), 0x3C00, dtype=np.uint16)
    got = oracle.bmm(wl.bits(P), ones, oracle.F16)
    # sequential fp64 sum over k, the same order -> identical bits
    Pv = _vals(P)
    want = np.zeros((b, L))
    for k in range(L):
        want += Pv[:, :, k]
    assert np.array_equal(got, np.repeat(want[:, :, None], d, axis=2))
    assert np.max(np.abs(want - 1.0)) < 5e-3                       # softmax rows sum to ~1
    # one-hot rows of P gather rows of V exactly
    V = wl.normal((b, L, d), "f16", 23, 0.125)
    idx = np.random.default_rng(0).integers(0, L, size=(b, L))
    H = np.zeros((b, L, L), dtype=np.uint16)
    for i in range(b):
        H[i, np.arange(L), idx[i]] = 0x3C00
    got = oracle.bmm(H, wl.bits(V), oracle.F16)
    for i in range(b):
        assert np.array_equal(got[i], _vals(V[i])[idx[i]])


# ---- fused elementwise epilogue --------------------------------------------------------------
def test_epilogue_closed_forms():
    C = np.array([[-2.0, 0.0, 3.0], [4.0, -5.0, 6.0]])
    assert np.array_equal(oracle.epilogue(C), C)                                   # identity
    assert np.array_equal(oracle.epilogue(C, 1.0, None, 1), np.array([[0, 0, 3.0], [4.0, 0, 6.0]]))
    assert np.array_equal(oracle.epilogue(C, 0.5, [1.0, 2.0, 3.0], 0),
                          np.array([[0.0, 2.0, 4.5], [3.0, -0.5, 6.0]]))           # bias per column
    assert np.array_equal(oracle.epilogue(C, -1.0, [0.0, 0.0, 0.0], 1), np.array([[2.0, 0, 0], [0, 5.0, 0]]))
    # relu(x) - relu(-x) = x
    assert np.array_equal(oracle.epilogue(C, 1.0, None, 1) - oracle.epilogue(C, -1.0, None, 1), C)
