// Launcher and table helpers of the persistent producer / consumer kernels; included by their
// instance shard only, so that work on that kernel does not recompile the other shards.
#pragma once
#include "alcop_instantiate.hip.h"
#include "alcop_stream.hip.h"

namespace alcop {

// Persistent producer / consumer kernels (schedule variant 2).
template <class C>
hipError_t prepare_stream()
{
  static std::once_flag once;
  static hipError_t attr_rc = hipSuccess;
  std::call_once(once, [] {
    attr_rc = hipFuncSetAttribute((const void*)alcop_stream<C, Gfx950>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
  });
  return attr_rc;
}

template <class C>
hipError_t launch_stream(const Params& p, dim3 grid, hipStream_t st)
{
  const hipError_t rc = prepare_stream<C>();
  if (rc != hipSuccess) return rc;
  alcop_stream<C, Gfx950><<<grid, dim3(C::NT), C::LDS_BYTES, st>>>(p);
  return hipGetLastError();
}

constexpr bool stream_feasible(int bm, int bn, int bk, int wm, int wn, int s)
{
  const int waves = (bm / wm) * (bn / wn);
  const int a = bm * bk * 2, b = bn * bk * 2;
  if (waves != 4) return false;
  if (a % (256 * 16) || b % (256 * 16)) return false;
  if (s * (a + b) + waves * 32 * (wn * 4 + 16) > 160 * 1024) return false;
  if ((s - 2) * ((a + b) / (256 * 16)) > 63) return false;
  return s >= 2 && s <= 4;
}

template <int DT, int BM, int BN, int BK, int WM, int WN, int S, int BL, int AM, int AL = 0, int FU = 1>
void add_stream(std::vector<KernelEntry>& t)
{
  if constexpr (stream_feasible(BM, BN, BK, WM, WN, S) && (FU != 2 || BK >= 64)) {
    using C = SCfg<DT, BM, BN, BK, WM, WN, S, BL, AM, AL, FU>;
    // FU = 2, the deep register pipeline of the consumers, is named reg_stages = 4 (fused) by the schedules
    t.push_back(KernelEntry{DT, BM, BN, BK, WM, WN, S, FU == 2 ? 4 : 2, FU ? 1 : 0, BL, AM, AL, 0, 0, 1, C::LDS_BYTES, C::NT,
                            C::L, 0, &launch_stream<C>, &prepare_stream<C>});
  }
}

}  // namespace alcop

// every ring depth, the consumers' register pipeline fused across k-tiles and not
#define ALCOP_STREAM_STAGES(T, DT, BM, BN, BK, WM, WN, BL, AM)   \
  add_stream<DT, BM, BN, BK, WM, WN, 2, BL, AM, 0, 1>(T);        \
  add_stream<DT, BM, BN, BK, WM, WN, 3, BL, AM, 0, 1>(T);        \
  add_stream<DT, BM, BN, BK, WM, WN, 4, BL, AM, 0, 1>(T);        \
  add_stream<DT, BM, BN, BK, WM, WN, 2, BL, AM, 0, 0>(T);        \
  add_stream<DT, BM, BN, BK, WM, WN, 3, BL, AM, 0, 0>(T);        \
  add_stream<DT, BM, BN, BK, WM, WN, 4, BL, AM, 0, 0>(T);
// the consumers' deep register pipeline (k-tile 64): measured no faster than the two above on any
// configuration, so these stay outside the default schedule space (alcop_sched_variants)
#define ALCOP_STREAM_DEEP(T, DT, BM, BN, WM, WN, BL, AM)         \
  add_stream<DT, BM, BN, 64, WM, WN, 2, BL, AM, 0, 2>(T);        \
  add_stream<DT, BM, BN, 64, WM, WN, 3, BL, AM, 0, 2>(T);
