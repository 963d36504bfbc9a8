// Helpers used by the instance shards: launcher template and cartesian-product macros.
#pragma once
#include <mutex>

#include "alcop_gfx950.hip.h"
#include "alcop_registry.h"

namespace alcop {

// LDS rings above the default 64 KB per-block limit need an explicit opt-in (the patch
// convolution sizes its LDS per call, up to the 160 KB a block can have).  Once per kernel and
// process; concurrent first callers wait for the one that sets it.
template <class C>
hipError_t prepare_instance()
{
  static std::once_flag once;
  static hipError_t attr_rc = hipSuccess;
  std::call_once(once, [] {
    attr_rc = hipFuncSetAttribute((const void*)alcop_mainloop<C, Gfx950>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize,
                                  C::AM == 3 ? 160 * 1024 : C::LDS_BYTES);
  });
  return attr_rc;
}

template <class C>
hipError_t launch_instance(const Params& p, dim3 grid, hipStream_t st)
{
  const hipError_t rc = prepare_instance<C>();
  if (rc != hipSuccess) return rc;
  alcop_mainloop<C, Gfx950><<<grid, dim3(C::NT), dynamic_lds_bytes<C>(p), st>>>(p);
  return hipGetLastError();
}

constexpr bool instance_feasible(int bm, int bn, int bk, int wm, int wn, int s, int r, int f,
                                 int pf = 0)
{
  const int nt = (bm / wm) * (bn / wn) * 64;
  const int a = bm * bk * 2, b = bn * bk * 2;
  if (a % (nt * 16) || b % (nt * 16)) return false;
  if (s * (a + b) + (pf ? (nt / 64) * 256 : 0) > 160 * 1024) return false;
  if (f && (r < 2 || s < 2)) return false;
  if (r > 2 && (!f || (r - 1) * 16 > bk)) return false;
  const int l = (a + b) / (nt * 16) + pf;
  if (s >= 2 && (s - 2) * l > 63) return false;
  return true;
}

template <int DT, int BM, int BN, int BK, int WM, int WN, int S, int R, int F, int BL, int AM,
          int AL = 0, int SK = 0, int PF = 0>
void add_instance(std::vector<KernelEntry>& t)
{
  if constexpr (instance_feasible(BM, BN, BK, WM, WN, S, R, F, PF)) {
    using C = KCfg<DT, BM, BN, BK, WM, WN, S, R, F, BL, AM, AL, SK, PF>;
    t.push_back(KernelEntry{DT, BM, BN, BK, WM, WN, S, R, F, BL, AM, AL, SK, PF, 0, C::LDS_BYTES, C::NT,
                            C::L, C::PATCH_OFF, &launch_instance<C>, &prepare_instance<C>});
  }
}

}  // namespace alcop

// Every pipelining variant of one tile: S in 1..4 single-level (R=1), multi-level unfused
// (R=2), multi-level fused (R=2, F=1).  Infeasible combinations are skipped at compile time.
#define ALCOP_ALL_PIPES(T, DT, BM, BN, BK, WM, WN, BL, AM)      \
  add_instance<DT, BM, BN, BK, WM, WN, 1, 1, 0, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 2, 1, 0, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 1, 0, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 4, 1, 0, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 1, 2, 0, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 2, 2, 0, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 2, 0, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 4, 2, 0, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 2, 2, 1, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 2, 1, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 4, 2, 1, BL, AM>(T);

// A reduced set: the unpipelined baseline, double buffering, and the fused multi-level ones.
#define ALCOP_KEY_PIPES(T, DT, BM, BN, BK, WM, WN, BL, AM)      \
  add_instance<DT, BM, BN, BK, WM, WN, 1, 1, 0, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 2, 1, 0, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 1, 0, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 2, 2, 1, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 2, 1, BL, AM>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 4, 2, 1, BL, AM>(T);

// The same reduced set for A stored K x M (transA).
#define ALCOP_KEY_PIPES_TA(T, DT, BM, BN, BK, WM, WN, BL)          \
  add_instance<DT, BM, BN, BK, WM, WN, 1, 1, 0, BL, 0, 1>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 2, 1, 0, BL, 0, 1>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 1, 0, BL, 0, 1>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 2, 2, 1, BL, 0, 1>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 2, 1, BL, 0, 1>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 4, 2, 1, BL, 0, 1>(T);

// Split-K variants: the unpipelined baseline and the fused multi-level pipelines.
#define ALCOP_SPLITK_PIPES(T, DT, BM, BN, BK, WM, WN, BL, AM)         \
  add_instance<DT, BM, BN, BK, WM, WN, 1, 1, 0, BL, AM, 0, 1>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 2, 2, 1, BL, AM, 0, 1>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 2, 1, BL, AM, 0, 1>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 4, 2, 1, BL, AM, 0, 1>(T);

// The same for A stored K x M (the layout of a weight-gradient product X^T . dY, whose output is
// small and whose reduction axis is the long batch axis).
#define ALCOP_SPLITK_PIPES_TA(T, DT, BM, BN, BK, WM, WN, BL)          \
  add_instance<DT, BM, BN, BK, WM, WN, 1, 1, 0, BL, 0, 1, 1>(T);       \
  add_instance<DT, BM, BN, BK, WM, WN, 2, 2, 1, BL, 0, 1, 1>(T);       \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 2, 1, BL, 0, 1, 1>(T);       \
  add_instance<DT, BM, BN, BK, WM, WN, 4, 2, 1, BL, 0, 1, 1>(T);

#define ALCOP_BOTH_BK(MACRO, T, DT, BM, BN, WM, WN, BL, AM) \
  MACRO(T, DT, BM, BN, 32, WM, WN, BL, AM)                  \
  MACRO(T, DT, BM, BN, 64, WM, WN, BL, AM)
