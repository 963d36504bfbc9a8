"""Host-side checks that need no GPU: the shared library loads and exports every symbol that
include/alcop.h declares; argument validation returns error codes before any launch; the
schedule space and feasibility rules."""
import ctypes
import os
import re

import pytest

import paper_2210_16691_amd as al

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "alcop.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(alcop_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert set(names) == set(al.EXPORTS)
    L = al.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_strerror():
    assert "gfx950" in al.version()
    assert al.strerror(0) == "ok"
    for code in range(-9, 0):
        assert al.strerror(code) != "unknown status"
    assert al.strerror(-99) == "unknown status"


def test_init_reports_a_missing_device_as_an_error():
    # on a machine without a GPU the kernels cannot be opted in to their LDS size; with one it succeeds
    assert al.lib().alcop_init() in (al.OK, al.ERR_LAUNCH)


def test_null_and_bad_arguments_are_rejected_without_a_launch():
    L = al.lib()
    s = al.sched(128, 128, 64, 64, 64, 1, 1, 0)
    fake = ctypes.c_void_p(0x10000)           # never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x10008)
    g = lambda A, B, C, M, N, K, lda, ldb, ldc, tA, tB, i, o: L.alcop_gemm(
        A, B, C, M, N, K, lda, ldb, ldc, tA, tB, i, o, ctypes.byref(s), None)
    assert g(None, fake, fake, 128, 128, 64, 64, 128, 128, 0, 0, 0, 0) == al.ERR_NULL
    assert g(fake, fake, None, 128, 128, 64, 64, 128, 128, 0, 0, 0, 0) == al.ERR_NULL
    assert g(fake, fake, fake, 128, 128, 64, 64, 128, 128, 1, 0, 0, 0) == al.ERR_SHAPE   # transA: lda < M
    assert g(fake, fake, fake, 100, 128, 64, 104, 128, 128, 1, 0, 0, 0) == al.ERR_SHAPE  # transA: M % 8
    assert g(fake, fake, fake, 128, 128, 64, 64, 128, 128, 0, 0, 2, 0) == al.ERR_DTYPE
    assert g(fake, fake, fake, 128, 128, 64, 64, 128, 128, 0, 0, 0, 7) == al.ERR_DTYPE
    assert g(fake, fake, fake, 0, 128, 64, 64, 128, 128, 0, 0, 0, 0) == al.ERR_SHAPE
    assert g(fake, fake, fake, 128, 100, 64, 64, 104, 104, 0, 0, 0, 0) == al.ERR_SHAPE   # N % 8
    assert g(odd, fake, fake, 128, 128, 64, 64, 128, 128, 0, 0, 0, 0) == al.ERR_ALIGN
    assert g(fake, fake, fake, 128, 128, 64, 68, 128, 128, 0, 0, 0, 0) == al.ERR_ALIGN   # lda % 8
    assert g(fake, fake, fake, 128, 128, 64, 56, 128, 128, 0, 0, 0, 0) == al.ERR_SHAPE   # lda < K
    assert g(fake, fake, fake, 128, 128, 100, 104, 128, 128, 0, 0, 0, 0) == al.ERR_SHAPE  # K % 8
    bad = al.sched(128, 128, 64, 64, 64, 1, 2, 1)      # fusion needs S >= 2
    assert L.alcop_gemm(fake, fake, fake, 128, 128, 64, 64, 128, 128, 0, 0, 0, 0,
                        ctypes.byref(bad), None) == al.ERR_SCHED
    assert L.alcop_conv2d_igemm(fake, fake, fake, 1, 8, 8, 64, 64, 3, 3, 0, 1, 1, 1, 0, 0,
                                None, None) == al.ERR_SHAPE       # stride 0
    assert L.alcop_conv2d_igemm(fake, fake, fake, 1, 2, 2, 64, 64, 5, 5, 1, 1, 0, 0, 0, 0,
                                None, None) == al.ERR_SHAPE       # filter larger than image


def test_spans_strides_and_invalid_problems():
    L = al.lib()
    fake = ctypes.c_void_p(0x10000)
    s = al.sched(128, 128, 64, 64, 64, 2, 2, 1)
    bmm = lambda sA, sB, sC: L.alcop_bmm(fake, fake, fake, 4, 128, 128, 64, 64, 128, 128, sA, sB, sC,
                                         0, 0, 0, 0, ctypes.byref(s), None)
    assert bmm(-8192, 8192, 16384) == al.ERR_SHAPE            # a stride that walks backwards
    assert bmm(8192, 8196, 16384) == al.ERR_ALIGN
    # B stored K x N with a partial last k-tile: its rows k = K .. 63 are addressed past the
    # operand, (64 - 1) * ldb * 2 bytes must stay below 2 GiB although (K - 1) * ldb * 2 does
    ldb = 1 << 25
    g = lambda K: L.alcop_gemm(fake, fake, fake, 128, 128, K, 64, ldb, 128, 0, 0, 0, 0,
                               ctypes.byref(s), None)
    assert 2 * (24 - 1) * ldb < 2 ** 31 <= 2 * (64 - 1) * ldb
    assert g(24) == al.ERR_SIZE
    # the same rule for A stored K x M
    assert L.alcop_gemm(fake, fake, fake, 128, 128, 24, 1 << 25, 128, 128, 1, 0, 0, 0,
                        ctypes.byref(al.sched(128, 128, 64, 64, 64, 3, 2, 1)), None) == al.ERR_SIZE
    bad = al.problem(al.OP_GEMM, 128, 100, 64, al.F16, al.F16)
    with pytest.raises(al.AlcopError) as e:
        al.alcop_sched_space(bad)
    assert e.value.code == al.ERR_SHAPE


def test_feasibility_rules():
    p = al.problem(al.OP_GEMM, 2048, 2048, 2048, al.F16, al.F16)
    ok = al.sched(128, 128, 64, 64, 64, 3, 2, 1)
    assert al.alcop_sched_supported(p, ok) == al.OK
    # 256x256x64 needs 64 KB per stage: three stages exceed the 160 KB LDS -> not built, infeasible
    assert al.alcop_sched_supported(p, al.sched(256, 256, 64, 128, 128, 3, 2, 1)) == al.ERR_SCHED
    assert al.alcop_sched_supported(p, al.sched(256, 256, 64, 128, 128, 2, 2, 1)) == al.OK
    assert al.alcop_sched_supported(p, al.sched(128, 128, 64, 64, 64, 2, 1, 1)) == al.ERR_SCHED
    assert al.alcop_sched_supported(p, al.sched(128, 128, 48, 64, 64, 2, 1, 0)) == al.ERR_SCHED
    p2 = al.problem(al.OP_GEMM, 2048, 2048, 2080, al.F16, al.F16)       # partial last k-tile: allowed
    assert al.alcop_sched_supported(p2, ok) == al.OK
    assert al.alcop_sched_supported(al.problem(al.OP_GEMM, 64, 64, 100, al.F16, al.F16), ok) == al.ERR_SHAPE
    pc = al.problem(al.OP_CONV2D, 32 * 56 * 56, 64, 576, al.F16, al.F16, conv_C=64)
    assert al.alcop_sched_supported(pc, al.sched(128, 64, 64, 64, 32, 3, 2, 1)) == al.OK
    pc32 = al.problem(al.OP_CONV2D, 1024, 64, 9 * 32, al.F16, al.F16, conv_C=32)
    # C = 32 with bk = 64: a k-tile spans two filter taps -> the per-lane gather kernels serve it
    assert al.alcop_sched_supported(pc32, al.sched(128, 64, 64, 64, 32, 3, 2, 1)) == al.OK
    assert al.alcop_sched_supported(pc32, al.sched(128, 64, 32, 64, 32, 3, 2, 1)) == al.OK
    # ... for fewer tiles than the one-tap gather is built for
    assert al.alcop_sched_supported(pc32, al.sched(64, 128, 64, 32, 64, 3, 2, 1)) == al.ERR_SCHED
    pc8 = al.problem(al.OP_CONV2D, 12544, 64, 49 * 8, al.F16, al.F16, conv_C=8)     # a padded RGB stem
    assert len([s for s in al.alcop_sched_space(pc8) if al.alcop_sched_supported(pc8, s) == al.OK]) >= 12
    assert al.alcop_sched_supported(al.problem(al.OP_CONV2D, 1024, 64, 9 * 12, al.F16, al.F16, conv_C=12),
                                    al.sched(128, 64, 32, 64, 32, 3, 2, 1)) == al.ERR_SHAPE


def test_sweep_of_the_motivating_example_is_built():
    # tile {64,128,256}^2 x k-tile {32,64} x stages {1..4}: 24 points, two exceed the LDS
    p = al.problem(al.OP_GEMM, 2048, 2048, 2048, al.F16, al.F16)
    space = {s.key()[:8] for s in al.alcop_sched_space(p)}
    waves = {64: 32, 128: 64, 256: 128}
    feasible = 0
    for b in (64, 128, 256):
        for bk in (32, 64):
            for S in (1, 2, 3, 4):
                lds = S * 2 * b * bk * 2
                has = any((b, b, bk, waves[b], waves[b], S, r, f) in space for r in (1, 2) for f in (0, 1))
                assert has == (lds <= 160 * 1024), (b, bk, S)
                feasible += has
    assert feasible == 22


def test_space_is_not_empty_for_every_operator():
    for p in [al.problem(al.OP_GEMM, 512, 512, 512, al.BF16, al.BF16),
              al.problem(al.OP_BMM, 512, 512, 64, al.F16, al.F16, batch=96, transB=True),
              al.problem(al.OP_BMM, 512, 64, 512, al.F16, al.F16, batch=96),
              al.problem(al.OP_CONV2D, 6272, 256, 2304, al.F16, al.F16, conv_C=256)]:
        sp = al.alcop_sched_space(p)
        assert len(sp) >= 6
        assert any(al.alcop_sched_supported(p, s) == al.OK for s in sp)


def test_ctypes_mirrors_match_the_c_structs(tmp_path):
    # compile a tiny C program against include/alcop.h and compare sizes / field offsets
    import subprocess
    src = tmp_path / "layout.c"
    src.write_text(r'''
#include <stdio.h>
#include <stddef.h>
#include "alcop.h"
int main(void) {
  printf("%zu %zu %zu\n", sizeof(alcop_sched), sizeof(alcop_problem), sizeof(alcop_epilogue));
  printf("%zu %zu %zu\n", offsetof(alcop_sched, l2_prefetch), offsetof(alcop_problem, transA),
         offsetof(alcop_epilogue, act));
  printf("%zu %zu %zu\n", offsetof(alcop_problem, conv_C), offsetof(alcop_epilogue, bias), offsetof(alcop_sched, variant));
  return 0;
}''')
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    out = subprocess.check_output([str(exe)]).decode().split()
    got = [int(v) for v in out]
    want = [ctypes.sizeof(al.Sched), ctypes.sizeof(al.Problem), ctypes.sizeof(al.Epilogue),
            al.Sched.l2_prefetch.offset, al.Problem.transA.offset, al.Epilogue.act.offset,
            al.Problem.conv_C.offset, al.Epilogue.bias.offset, al.Sched.variant.offset]
    assert got == want


def test_model_prefers_pipelining_and_large_tiles_on_a_large_square():
    # sanity of the ranking on 8192^3: a multi-stage 256x256 schedule is predicted faster than its
    # own 1-stage version and than any 64x64 schedule
    p = al.problem(al.OP_GEMM, 8192, 8192, 8192, al.BF16, al.BF16)
    t = lambda s: al.alcop_model_predict(p, s, 0)[0]
    big = t(al.sched(256, 256, 32, 128, 64, 4, 2, 1))
    assert big < t(al.sched(256, 256, 32, 128, 64, 1, 1, 0))
    assert big < min(t(s) for s in al.alcop_sched_space(p) if s.bm == 64 and s.bn == 64)
    # every prediction is finite and positive, for both models
    for s in al.alcop_sched_space(p):
        for m in (0, 1):
            v = t(s) if m == 0 else al.alcop_model_predict(p, s, 1)[0]
            assert v > 0 and v < 1e9


def test_auto_schedule_is_the_models_top_one_and_cache_round_trip(tmp_path):
    p = al.problem(al.OP_GEMM, 1536, 1024, 768, al.BF16, al.BF16)
    feas = [s for s in al.alcop_sched_space(p) if al.alcop_sched_supported(p, s) == al.OK]
    best = min(feas, key=lambda s: al.alcop_model_predict(p, s, 0)[0])
    auto = al.alcop_sched_auto(p)
    assert al.alcop_model_predict(p, auto, 0)[0] == al.alcop_model_predict(p, best, 0)[0]
    # a cache file overrides the model's pick; lines that cannot run are ignored
    f = tmp_path / "cache.txt"
    f.write_text(
        "0 1 1536 1024 768 0 0 1 1 0 : 64 64 32 32 32 2 2 1 1 0\n"      # valid
        "0 1 1536 1024 768 0 0 1 1 0 : 96 64 32 32 32 2 2 1 1 0\n"      # no such kernel
        "0 1 1000 1001 768 0 0 1 1 0 : 64 64 32 32 32 2 2 1 1 0\n"      # N % 8 != 0
        "garbage\n")
    assert al.alcop_cache_load(str(f)) == 1
    assert al.alcop_sched_auto(p).key() == (64, 64, 32, 32, 32, 2, 2, 1, 1, 0, 0)
    out = tmp_path / "saved.txt"
    n = al.alcop_cache_save(str(out))
    assert n >= 1
    assert "0 1 1536 1024 768 0 0 1 1 0 : 64 64 32 32 32 2 2 1 1 0" in out.read_text()
    with pytest.raises(al.AlcopError) as e:
        al.alcop_cache_load(str(tmp_path / "missing.txt"))
    assert e.value.code == al.ERR_IO


def test_splitk_space_model_pick_and_argument_checks():
    L = al.lib()
    rn50 = al.problem(al.OP_GEMM, 1024, 64, 2048, al.F16, al.F16)          # 16 tiles of 64 x 64
    big = al.problem(al.OP_GEMM, 8192, 8192, 8192, al.BF16, al.BF16)
    conv = al.problem(al.OP_CONV2D, 6272, 256, 2304, al.F16, al.F16, conv_C=256)
    for p in (rn50, big, conv, al.problem(al.OP_GEMM, 512, 512, 512, al.BF16, al.F32, transB=True)):
        assert len(al.alcop_splitk_space(p)) >= 4
    s, split, us = al.alcop_splitk_auto(rn50)
    assert split >= 4
    assert us < al.alcop_model_predict(rn50, al.alcop_sched_auto(rn50), 0)[0]
    assert al.alcop_splitk_auto(big)[1] == 1          # plenty of tiles: slicing only adds a pass
    assert al.alcop_splitk_auto(conv)[1] >= 1         # 98 tiles: measured, slicing does not pay here
    # more slices than k-tiles are clamped by the launch, not by the query; the query is monotone
    # in nothing in particular, but every answer is a built variant
    keys = {v.key() for v in al.alcop_splitk_space(rn50)}
    for k in (1, 2, 8, 64):
        assert al.alcop_splitk_auto(rn50, k)[0].key() in keys
    assert al.alcop_splitk_workspace_bytes(2, 128, 64, 3) == 4 * 3 * 2 * 128 * 64
    assert al.alcop_splitk_workspace_bytes(1, 128, 64, 0) == 0
    fake = ctypes.c_void_p(0x10000)
    call = lambda tA, split, ws, nbytes: L.alcop_gemm_splitk(
        fake, fake, fake, 1, 128, 64, 512, 512, 64, 64, 0, 0, 0, tA, 0, 0, 0, None, None, split,
        ws, nbytes, None)
    # A stored K x M together with B stored N x K: no split-K variant is built for that pair
    assert L.alcop_gemm_splitk(fake, fake, fake, 1, 128, 64, 512, 128, 512, 64, 0, 0, 0, 1, 1, 0, 0,
                               None, None, 2, fake, 1 << 20, None) == al.ERR_SCHED
    assert call(0, 2, None, 1 << 20) == al.ERR_NULL
    assert call(0, 2, ctypes.c_void_p(0x10004), 1 << 20) == al.ERR_ALIGN
    assert call(0, -1, fake, 1 << 20) == al.ERR_SHAPE
    assert call(0, 2, fake, 4 * 2 * 128 * 64 - 1) == al.ERR_SIZE
    best, k, us = al.Sched(), ctypes.c_int(), ctypes.c_double()
    tune = lambda ws, top_k: L.alcop_tune_splitk(
        ctypes.byref(rn50), fake, fake, fake, 2048, 64, 64, 0, 0, 0, None, ws, 1 << 20, top_k, 5,
        ctypes.byref(best), ctypes.byref(k), ctypes.byref(us), None, None, None, None, None, None, 0, None)
    assert tune(None, 5) == al.ERR_NULL
    assert tune(fake, -1) == al.ERR_SHAPE


def test_tuning_cache_named_by_the_environment(tmp_path):
    import subprocess
    import sys
    f = tmp_path / "cache.txt"
    f.write_text("0 1 1536 1024 768 0 0 1 1 0 : 64 64 32 32 32 2 2 1 1 0\n")
    code = ("import paper_2210_16691_amd as al\n"
            "p = al.problem(al.OP_GEMM, 1536, 1024, 768, al.BF16, al.BF16)\n"
            "print(al.alcop_sched_auto(p).key())\n")
    env = dict(os.environ, ALCOP_TUNE_CACHE=str(f), PYTHONPATH=ROOT)
    out = subprocess.check_output([sys.executable, "-c", code], env=env, cwd=ROOT).decode()
    assert out.strip() == "(64, 64, 32, 32, 32, 2, 2, 1, 1, 0, 0)"
    env["ALCOP_TUNE_CACHE"] = str(tmp_path / "missing.txt")          # ignored, the model decides
    out = subprocess.check_output([sys.executable, "-c", code], env=env, cwd=ROOT).decode()
    assert out.strip() != "(64, 64, 32, 32, 32, 2, 2, 1, 1, 0, 0)"


def test_binding_rejects_mismatched_operands_before_the_c_call():
    # the library sizes its buffer descriptors from the shapes it is told; the binding must not
    # tell it shapes the tensors do not have (CPU tensors here: nothing may reach the C call)
    import torch
    f16, f32 = torch.float16, torch.float32
    A, B, C = torch.zeros(128, 64, dtype=f16), torch.zeros(64, 136, dtype=f16), torch.zeros(128, 136, dtype=f16)
    s = al.sched(128, 128, 64, 64, 64, 1, 1, 0)
    with pytest.raises(ValueError, match="reduction extents"):
        al.alcop_gemm(A, torch.zeros(56, 136, dtype=f16), C, s)
    with pytest.raises(ValueError, match="reduction extents"):
        al.alcop_gemm(A, B, torch.zeros(128, 64, dtype=f16), s, transB=True)     # B read as [N, K]: K = 136
    with pytest.raises(ValueError, match="C is"):
        al.alcop_gemm(A, B, torch.zeros(128, 128, dtype=f16), s)
    with pytest.raises(ValueError, match="dtype"):
        al.alcop_gemm(A, B.to(torch.bfloat16), C, s)
    with pytest.raises(ValueError, match="contiguous"):
        al.alcop_gemm(torch.zeros(64, 128, dtype=f16).t(), B, C, s)
    with pytest.raises(ValueError, match="2-D"):
        al.alcop_gemm(A[None], B[None], C[None], s)
    with pytest.raises(KeyError):
        al.alcop_gemm(A, B, C.to(torch.float64), s)
    Ab, Bb, Cb = A[None].repeat(3, 1, 1), B[None].repeat(2, 1, 1), C[None].repeat(3, 1, 1)
    with pytest.raises(ValueError, match="batch sizes"):
        al.alcop_bmm(Ab, Bb, Cb, s)
    with pytest.raises(ValueError, match="bias"):
        al.alcop_gemm_fused(A, B, C, 1.0, torch.zeros(128, dtype=f32), 0, s)
    with pytest.raises(ValueError, match="reduction extents"):
        al.alcop_gemm_splitk(A, torch.zeros(72, 136, dtype=f16), C, 2, torch.zeros(1 << 16), s)
    x, w = torch.zeros(2, 8, 8, 64, dtype=f16), torch.zeros(3, 3, 64, 32, dtype=f16)
    with pytest.raises(ValueError, match="y is"):
        al.alcop_conv2d_igemm(x, w, torch.zeros(2, 8, 8, 64, dtype=f16), (1, 1), (1, 1))
    with pytest.raises(ValueError, match="y is"):
        al.alcop_conv2d_igemm(x, w, torch.zeros(2, 8, 8, 32, dtype=f16), (1, 1), (0, 0))   # 6 x 6 without padding
    with pytest.raises(ValueError, match="channel counts"):
        al.alcop_conv2d_igemm(x, torch.zeros(3, 3, 32, 32, dtype=f16), torch.zeros(2, 8, 8, 32, dtype=f16), (1, 1), (1, 1))
    with pytest.raises(ValueError, match="channel counts"):
        al.alcop_conv2d_igemm_krsc(x, w, torch.zeros(2, 8, 8, 3, dtype=f16), (1, 1), (1, 1))  # w read as KRSC: C = 32
    with pytest.raises(ValueError, match="contiguous"):
        al.alcop_conv2d_igemm(x.permute(0, 2, 1, 3), w, torch.zeros(2, 8, 8, 32, dtype=f16), (1, 1), (1, 1))


def test_diagnostic_library_exports_what_its_header_declares():
    from paper_2210_16691_amd import diag
    text = open(os.path.join(ROOT, "include", "alcop_diag.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(alcop_diag_[a-z0-9_]+)\s*\(", text)))
    assert set(names) == set(diag.EXPORTS)
    L = diag.lib()
    for n in names:
        assert getattr(L, n) is not None
    cfgs = diag.configs()
    assert len(cfgs) >= 3 and all(c.split()[0] in ("f16", "bf16") for c in cfgs)
    assert L.alcop_diag_config_name(len(cfgs)) is None


def test_ranked_order_is_the_model_order_with_a_cap_per_tile_family():
    prob = al.problem(al.OP_BMM, 512, 64, 512, al.F16, al.F16, batch=96)
    space = [s for s in al.alcop_sched_space(prob) if al.alcop_sched_supported(prob, s) == al.OK]
    ranked = al.alcop_sched_ranked(prob, 0, False, 10)
    assert sorted(s.key() for s in ranked) == sorted(s.key() for s in space)      # a permutation of the space
    fam = lambda s: (s.bm, s.bn, s.bk, s.wm, s.wn, s.variant)
    pred = lambda s: al.alcop_model_predict(prob, s, 0)[0]
    head = ranked[:10]
    counts = {}
    for s in head:
        counts[fam(s)] = counts.get(fam(s), 0) + 1
    assert max(counts.values()) <= 3 and len(counts) >= 4
    # the one-stage schedule of the two best-ranked tile-at-a-time families closes the budget
    plain_fams = []
    for s in head:
        if s.variant == 0 and fam(s) not in plain_fams:
            plain_fams.append(fam(s))
    for f in plain_fams[:2]:
        assert any(fam(s) == f and s.stages == 1 for s in head), f
    insured = [s for s in head if s.stages == 1 and fam(s) in plain_fams[:2]]
    rest = [s for s in head if s not in insured]
    # apart from those, within a family the head holds its best-predicted members, in model order
    for f in {fam(s) for s in rest}:
        members = sorted((pred(s) for s in space if fam(s) == f))
        mine = sorted(pred(s) for s in rest if fam(s) == f)
        assert mine == members[:len(mine)]
    assert [pred(s) for s in rest] == sorted(pred(s) for s in rest)
    assert head[-len(insured):] == insured or all(pred(s) <= pred(rest[-1]) for s in insured)
    # no budget: the plain model order
    plain = al.alcop_sched_ranked(prob, 0, False, 0)
    assert [pred(s) for s in plain] == sorted(pred(s) for s in plain)


def test_unaligned_entry_points_reject_bad_arguments_without_a_launch():
    L = al.lib()
    fake = ctypes.c_void_p(0x10000)           # never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x10001)
    ws = ctypes.c_void_p(0x20000)
    need = al.alcop_unaligned_workspace_bytes(2, 9, 10, 11, al.F32)
    # three padded images: 2 x 16 x 16 halves twice, 2 x 16 x 16 floats, and 16 floats of bias
    assert need == 1024 + 1024 + 2048 + 256

    def bmm(A, B, C, batch, M, N, K, lda, ldb, ldc, it, ot, w, wbytes, tA=0, tB=0):
        return L.alcop_bmm_unaligned(A, B, C, batch, M, N, K, lda, ldb, ldc, 200, 200, 200, tA, tB, it, ot,
                                     None, None, w, wbytes, None)
    assert bmm(None, fake, fake, 2, 9, 10, 11, 11, 10, 10, al.F16, al.F32, ws, need) == al.ERR_NULL
    assert bmm(fake, fake, fake, 2, 9, 10, 11, 11, 10, 10, al.F16, al.F32, None, need) == al.ERR_NULL
    assert bmm(fake, fake, fake, 2, 9, 10, 11, 11, 10, 10, al.F32, al.F32, ws, need) == al.ERR_DTYPE
    assert bmm(fake, fake, fake, 2, 9, 10, 11, 11, 10, 10, al.F16, 5, ws, need) == al.ERR_DTYPE
    assert bmm(fake, fake, fake, 2, 0, 10, 11, 11, 10, 10, al.F16, al.F32, ws, need) == al.ERR_SHAPE
    assert bmm(fake, fake, fake, 2, 9, 10, 11, 10, 10, 10, al.F16, al.F32, ws, need) == al.ERR_SHAPE   # lda < K
    assert bmm(fake, fake, fake, 2, 9, 10, 11, 11, 10, 9, al.F16, al.F32, ws, need) == al.ERR_SHAPE    # ldc < N
    assert bmm(fake, fake, fake, 2, 9, 10, 11, 8, 10, 10, al.F16, al.F32, ws, need, tA=1) == al.ERR_SHAPE  # A stored K x M: lda < M
    assert bmm(odd, fake, fake, 2, 9, 10, 11, 11, 10, 10, al.F16, al.F32, ws, need) == al.ERR_ALIGN
    assert bmm(fake, fake, ctypes.c_void_p(0x10002), 2, 9, 10, 11, 11, 10, 10, al.F16, al.F32, ws, need) == al.ERR_ALIGN
    assert bmm(fake, fake, fake, 2, 9, 10, 11, 11, 10, 10, al.F16, al.F32, ctypes.c_void_p(0x20008), need) == al.ERR_ALIGN
    assert bmm(fake, fake, fake, 2, 9, 10, 11, 11, 10, 10, al.F16, al.F32, ws, need - 1) == al.ERR_SIZE
    assert bmm(fake, fake, fake, 70000, 9, 10, 11, 11, 10, 10, al.F16, al.F32, ws, 1 << 40) == al.ERR_SHAPE

    def conv(x, w, y, C, K, wsp, wbytes, it=al.F16, stride=1, dil=1, H=6):
        return L.alcop_conv2d_igemm_unaligned(x, w, y, 2, H, 6, C, K, 3, 3, stride, stride, 1, 1, dil, dil, it, al.F16,
                                              None, None, wsp, wbytes, None)
    cneed = al.alcop_conv2d_unaligned_workspace_bytes(2, 6, 6, 3, 5, 3, 3, (1, 1), (1, 1), (1, 1), al.F16)
    # x: 72 pixels x 8 channels, w: 9 x 8 x 8, y: 72 x 8 (halves), bias 8 floats; 256-byte sections
    assert cneed == 1280 + 1280 + 1280 + 256
    assert conv(None, fake, fake, 3, 5, ws, cneed) == al.ERR_NULL
    assert conv(fake, fake, fake, 3, 5, ws, cneed, it=al.F32) == al.ERR_DTYPE
    assert conv(fake, fake, fake, 0, 5, ws, cneed) == al.ERR_SHAPE
    assert conv(fake, fake, fake, 3, 5, ws, cneed, stride=0) == al.ERR_SHAPE
    assert conv(fake, fake, fake, 3, 5, ws, cneed, dil=4, H=2) == al.ERR_SHAPE      # the dilated filter exceeds the padded image
    assert conv(odd, fake, fake, 3, 5, ws, cneed) == al.ERR_ALIGN
    assert conv(fake, fake, fake, 3, 5, ws, cneed - 1) == al.ERR_SIZE
