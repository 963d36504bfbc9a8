"""Address / undefined-behaviour sanitizer runs of the host-only native code: the C oracle and
the static model + measurement-corrected model.  (The GPU code cannot run under a sanitizer
here; its indexing is checked on the CPU model in test_emulated_kernel.py.)"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
# verify_asan_link_order=0: a preloaded library in the environment must not abort the run
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="halt_on_error=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=ENV, **kw)
    assert r.returncode == 0, r.stdout[-3000:]
    return r.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_under_sanitizers(tmp_path):
    drv = tmp_path / "drv.c"
    drv.write_text(r'''
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
int alcop_oracle_gemm(const uint16_t*, const uint16_t*, double*, int, int, int, long, long, long, int, int, int);
int alcop_oracle_bmm(const uint16_t*, const uint16_t*, double*, int, int, int, int, long, long, long, long, long, long, int, int, int);
int alcop_oracle_conv2d(const uint16_t*, const uint16_t*, double*, int, int, int, int, int, int, int, int, int, int, int, int);
double alcop_oracle_decode_f16(uint16_t);
double alcop_oracle_decode_bf16(uint16_t);
static uint16_t* fill(size_t n, unsigned seed) {
  uint16_t* p = malloc(n * 2);                       /* exactly n elements: one past is an error */
  for (size_t i = 0; i < n; i++) { seed = seed * 1664525u + 1013904223u; p[i] = (uint16_t)(0x3c00 + (seed >> 24)); }
  return p;
}
int main(void) {
  double acc = 0;
  for (unsigned h = 0; h < 65536; h++) { double a = alcop_oracle_decode_f16((uint16_t)h), b = alcop_oracle_decode_bf16((uint16_t)h); acc += (a == a ? 1 : 0) + (b == b ? 1 : 0); }
  for (int tA = 0; tA < 2; tA++) for (int tB = 0; tB < 2; tB++) for (int dt = 0; dt < 2; dt++) {
    int M = 37, N = 24, K = 19;
    uint16_t *A = fill((size_t)M * K, 1), *B = fill((size_t)K * N, 2);
    double* C = malloc(sizeof(double) * M * N);
    if (alcop_oracle_gemm(A, B, C, M, N, K, tA ? M : K, tB ? K : N, N, tA, tB, dt)) return 2;
    acc += C[M * N - 1];
    free(A); free(B); free(C);
  }
  { int b = 3, M = 9, N = 16, K = 8;
    uint16_t *A = fill((size_t)b * M * K, 3), *B = fill((size_t)b * K * N, 4);
    double* C = malloc(sizeof(double) * b * M * N);
    if (alcop_oracle_bmm(A, B, C, b, M, N, K, K, N, N, (long)M * K, (long)K * N, (long)M * N, 0, 0, 0)) return 3;
    acc += C[b * M * N - 1]; free(A); free(B); free(C); }
  { int N = 2, H = 7, W = 5, Cc = 8, K = 8, R = 3, S = 3, sh = 2, sw = 1, ph = 1, pw = 2;
    int P = (H + 2 * ph - R) / sh + 1, Q = (W + 2 * pw - S) / sw + 1;
    uint16_t *x = fill((size_t)N * H * W * Cc, 5), *w = fill((size_t)R * S * Cc * K, 6);
    double* y = malloc(sizeof(double) * N * P * Q * K);
    if (alcop_oracle_conv2d(x, w, y, N, H, W, Cc, K, R, S, sh, sw, ph, pw, 0)) return 4;
    acc += y[N * P * Q * K - 1]; free(x); free(w); free(y); }
  printf("ok %g\n", acc);
  return 0;
}''')
    exe = tmp_path / "oracle_san"
    _run(["gcc"] + SAN + ["-fopenmp", str(drv), os.path.join(ROOT, "oracle", "alcop_oracle.c"), "-lm", "-o", str(exe)])
    assert _run([str(exe)]).startswith("ok")


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_static_model_and_corrector_under_sanitizers(tmp_path):
    drv = tmp_path / "drv.cpp"
    drv.write_text(r'''
#include <cmath>
#include <cstdio>
#include "alcop_model.h"
using namespace alcop;
int main() {
  const Device dev;
  const int tiles[][5] = {{64, 64, 32, 32, 32}, {128, 128, 64, 64, 64}, {256, 256, 32, 128, 64}, {256, 64, 64, 64, 64}, {64, 128, 64, 32, 64}};
  const int shapes[][5] = {{1, 8, 8, 8, 0}, {1, 2048, 2048, 2048, 0}, {96, 512, 512, 64, 0}, {1, 1024, 64, 2048, 0}, {1, 100352, 64, 576, 64}, {1, 8192, 8192, 8192, 0}};
  double acc = 0;
  Corrector corr;
  int n = 0;
  for (auto& sh : shapes) for (auto& t : tiles) for (int S = 1; S <= 4; S++) for (int R = 1; R <= 2; R++) for (int tb = 0; tb < 2; tb++) {
    alcop_problem p{};
    p.op = sh[4] ? ALCOP_OP_CONV2D : (sh[0] > 1 ? ALCOP_OP_BMM : ALCOP_OP_GEMM);
    p.batch = sh[0]; p.M = sh[1]; p.N = sh[2]; p.K = sh[3]; p.conv_C = sh[4]; p.transB = tb; p.transA = tb && !sh[4];
    p.in = ALCOP_F16; p.out = tb ? ALCOP_F32 : ALCOP_F16;
    alcop_sched s{t[0], t[1], t[2], t[3], t[4], S, R, (R == 2 && S >= 2) ? 1 : 0, 1, tb ? 4 : 0};
    for (int model = 0; model < 2; model++) {
      ModelTerms mt;
      const double us = predict(p, s, model, dev, &mt);
      if (!(us > 0) || !std::isfinite(us)) { std::printf("bad prediction\n"); return 2; }
      acc += us;
    }
    double x[Corrector::D];
    Corrector::features(p, s, dev, x);
    corr.add(x, predict(p, s, 0, dev, nullptr) * (1.0 + 0.1 * (n % 5)));
    if (++n % 7 == 0) corr.fit();
    acc += corr.predict_log(x);
  }
  std::printf("ok %g %d\n", acc, n);
  return 0;
}''')
    exe = tmp_path / "model_san"
    csrc = os.path.join(ROOT, "paper_2210_16691_amd", "csrc")
    _run(["g++", "-std=c++17"] + SAN + ["-I", csrc, str(drv), os.path.join(csrc, "alcop_model.cpp"), "-o", str(exe)])
    assert _run([str(exe)]).startswith("ok")
