"""The model-ranked tuner on the GPU: search-space pruning, ranking orders, best-in-k properties."""
import pytest
import torch

import paper_2210_16691_amd as al
import workloads as wl
from gpu_util import DEV

pytestmark = pytest.mark.gpu


def _problem():
    M, N, K = 1024, 1024, 1024
    A = wl.uniform((M, K), "f16", 401).to(DEV)
    B = wl.uniform((K, N), "f16", 402).to(DEV)
    C = torch.empty(M, N, dtype=torch.float16, device=DEV)
    return al.problem(al.OP_GEMM, M, N, K, al.F16, al.F16), A, B, C


def test_pruned_space_and_trial_counts():
    prob, A, B, C = _problem()
    space = al.alcop_sched_space(prob)
    feasible = [s for s in space if al.alcop_sched_supported(prob, s) == al.OK]
    r = al.alcop_tune(prob, A, B, C, top_k=7, model=0, iters=5)
    assert r.space == len(feasible) and r.trials == 7 and len(r.log) == 7
    assert r.best_us == min(us for _, _, us in r.log)
    # analytical-only ranking: trials come in non-decreasing predicted time
    preds = [p for _, p, _ in r.log]
    assert preds == sorted(preds)
    for s, p, _ in r.log:
        assert p == pytest.approx(al.alcop_model_predict(prob, s, 0)[0], rel=1e-12)


def test_exhaustive_covers_the_space_and_top_k_is_a_prefix():
    prob, A, B, C = _problem()
    ex = al.alcop_tune(prob, A, B, C, top_k=0, model=0, iters=5)
    assert ex.trials == ex.space
    top = al.alcop_tune(prob, A, B, C, top_k=10, model=0, iters=5)
    # the ten trials are the head of the ranked order (model order, at most two schedules per tile
    # family), and that order without a budget is the exhaustive run's
    assert [s.key() for s, _, _ in top.log] == [s.key() for s in al.alcop_sched_ranked(prob, 0, False, 10)[:10]]
    assert [s.key() for s, _, _ in ex.log] == [s.key() for s in al.alcop_sched_ranked(prob, 0, False, 0)]
    assert top.best_us >= ex.best_us * 0.5
    # best-in-top-k is non-decreasing in k and reaches the exhaustive best at k = |space|
    best = ex.best_us
    prev = 0.0
    for k in (1, 5, 10, 50, ex.space):
        q = best / min(us for _, _, us in ex.log[:k])
        assert q <= 1.0 + 1e-12 and q >= prev - 1e-12
        prev = q
    assert prev == pytest.approx(1.0)


def test_corrected_model_starts_from_the_analytical_ranking():
    prob, A, B, C = _problem()
    r0 = al.alcop_tune(prob, A, B, C, top_k=3, model=0, iters=5)
    r2 = al.alcop_tune(prob, A, B, C, top_k=12, model=2, iters=5)
    # no measurements yet -> the first trials are the analytical model's first
    assert [s.key() for s, _, _ in r2.log[:2]] == [s.key() for s, _, _ in r0.log[:2]]
    keys = [s.key() for s, _, _ in r2.log]
    assert len(set(keys)) == len(keys) == 12          # never times a schedule twice
    assert r2.best_us == min(us for _, _, us in r2.log)


def test_grid_order_is_table_order():
    prob, A, B, C = _problem()
    r3 = al.alcop_tune(prob, A, B, C, top_k=6, model=3, iters=3)
    table = [s for s in al.alcop_sched_space(prob) if al.alcop_sched_supported(prob, s) == al.OK]
    assert [s.key() for s, _, _ in r3.log] == [s.key() for s in table[:6]]


def test_auto_schedule_uses_the_tuned_result():
    prob, A, B, C = _problem()
    r = al.alcop_tune(prob, A, B, C, top_k=5, model=0, iters=5)
    ref = torch.empty_like(C)
    al.alcop_gemm(A, B, ref, r.best)
    al.alcop_gemm(A, B, C, None)                      # picks the cached tuned schedule
    torch.cuda.synchronize()
    assert torch.equal(C.view(torch.int16), ref.view(torch.int16))
