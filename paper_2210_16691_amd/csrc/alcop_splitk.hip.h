// Second step of a split-K product: sums the fp32 partial tiles that the grid.z slices of the
// main loop left in the workspace, applies the consumer-side elementwise function and writes C.
//
// Why split K at all: the paper tunes tile sizes against the number of tiles ("inter-tile
// parallelism", Sec. 1 and Fig. 1) and notes that a small output with a long reduction axis
// gains most from pipelining; on 256 compute units such shapes (16 to 192 tiles) leave most of
// the machine idle whatever the tile.  Slicing the reduction axis multiplies the number of
// blocks; the price is this extra pass and a result that is no longer bit-identical to the
// unsplit schedule (the slices are added in ascending z, so it is still deterministic).
//
// Like the main loop, the kernel takes the hardware operations from a policy class.
#pragma once
#include <stdint.h>

#include "alcop_kernel.hip.h"

namespace alcop {

struct ReduceParams {
  const float* ws;   // [split][batch][M][N] fp32 partial products
  void* C;           // output, row stride ldc, batch stride strideC (elements)
  int M, N;
  int ldc;
  long strideC;
  int split;
  long zstride;      // elements between consecutive slices in ws (= batch * M * N)
  int out_dtype;     // 0 f16, 1 bf16, 2 f32
  float alpha;       // act(alpha * sum + bias[n])
  const float* bias;
  int act;
};

constexpr int REDUCE_THREADS = 256;

// One thread owns 8 consecutive n of one row m (N % 8 == 0): two 16-byte loads per slice and one
// (fp16 / bf16) or two (fp32) 16-byte stores.  grid.x covers M * N / 8 threads, grid.y = batch.
template <class HW>
__global__ void __launch_bounds__(REDUCE_THREADS) alcop_splitk_reduce(const ReduceParams p)
{
  const int n8 = p.N >> 3;
  const long idx = (long)HW::block_x() * REDUCE_THREADS + HW::wave_id() * 64 + HW::lane_id();
  if (idx >= (long)p.M * n8) return;
  const int m = (int)(idx / n8), n = (int)(idx - (long)m * n8) * 8;
  const int batch = (int)HW::block_y();
  const float* src = p.ws + ((long)batch * p.M + m) * p.N + n;
  f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
  for (int z = 0; z < p.split; z++) {
    const f32x4 a = HW::global_load_f32x4(src + (long)z * p.zstride);
    const f32x4 b = HW::global_load_f32x4(src + (long)z * p.zstride + 4);
#pragma unroll
    for (int e = 0; e < 4; e++) {
      lo[e] += a[e];
      hi[e] += b[e];
    }
  }
  if (p.alpha != 1.0f || p.bias != nullptr || p.act != 0) {
    f32x4 b0 = {0.f, 0.f, 0.f, 0.f}, b1 = {0.f, 0.f, 0.f, 0.f};
    if (p.bias != nullptr) {
      b0 = HW::global_load_f32x4(p.bias + n);
      b1 = HW::global_load_f32x4(p.bias + n + 4);
    }
#pragma unroll
    for (int e = 0; e < 4; e++) {
      const float t0 = lo[e] * p.alpha + b0[e], t1 = hi[e] * p.alpha + b1[e];
      lo[e] = (p.act == 1 && t0 < 0.f) ? 0.f : t0;
      hi[e] = (p.act == 1 && t1 < 0.f) ? 0.f : t1;
    }
  }
  auto store = [&](auto zero) {
    using OT = decltype(zero);
    char* dst = (char*)p.C + ((long)batch * p.strideC + (long)m * p.ldc + n) * sizeof(OT);
    if constexpr (sizeof(OT) == 4) {
      HW::global_store16(dst, __builtin_bit_cast(u32x4, lo));
      HW::global_store16(dst + 16, __builtin_bit_cast(u32x4, hi));
    } else {
      typedef OT ot8 __attribute__((ext_vector_type(8)));
      const ot8 h = {HW::template cvt<OT>(lo[0]), HW::template cvt<OT>(lo[1]),
                     HW::template cvt<OT>(lo[2]), HW::template cvt<OT>(lo[3]),
                     HW::template cvt<OT>(hi[0]), HW::template cvt<OT>(hi[1]),
                     HW::template cvt<OT>(hi[2]), HW::template cvt<OT>(hi[3])};
      HW::global_store16(dst, __builtin_bit_cast(u32x4, h));
    }
  };
  if (p.out_dtype == 2)
    store(0.0f);
  else if (p.out_dtype == 0)
    store((_Float16)0);
  else
    store((__bf16)0);
}

}  // namespace alcop
