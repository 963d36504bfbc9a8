// Operands whose shape or placement the pipelined loops cannot take as they are: N or K not a
// multiple of 8, row pitches or base addresses that are not 16-byte aligned, a channel count such
// as 3.  The loops move 16-byte chunks (paper Sec. 4.2: the asynchronous copies of a pipeline
// stage; here one buffer_load_dwordx4 ... lds per lane), so such operands are first copied into a
// workspace with every extent rounded up to 8 elements and the tail zero-filled, the product is
// computed there by the ordinary kernels, and the valid part of the result is copied out.
// Zero padding leaves every valid output element unchanged: the extra k terms are exact zeros.
//
// Like the main loops, the two kernels take the hardware operations from a policy class.
#pragma once
#include <stdint.h>

#include "alcop_kernel.hip.h"

namespace alcop {

struct PackParams {
  const void* src;
  void* dst;
  int rows, cols;        // extent of the valid data (both kernels)
  long s_batch, s_row;   // source strides in elements; grid.y = batch entry
  int rows_d, cols_d;    // extent of the padded image: pack writes all of it, unpack reads the
                         // valid part of it; cols_d * esize is a multiple of 16
  long d_batch, d_row;   // destination strides in elements
  int esize;             // bytes per element: 2 or 4
};

constexpr int PACK_THREADS = 256;

// dst[b][r][c] = r < rows && c < cols ? src[b][r][c] : 0 for r < rows_d, c < cols_d.  The source
// needs element alignment only (element-wise loads); the destination rows are 16-byte aligned and
// one thread writes one 16-byte chunk.  grid.x covers rows_d * cols_d * esize / 16 threads.
template <class HW>
__global__ void __launch_bounds__(PACK_THREADS) alcop_pack(const PackParams p)
{
  const int per = 16 / p.esize, cpr = p.cols_d / per;
  const long idx = (long)HW::block_x() * PACK_THREADS + HW::wave_id() * 64 + HW::lane_id();
  if (idx >= (long)p.rows_d * cpr) return;
  const int r = (int)(idx / cpr), c0 = (int)(idx - (long)r * cpr) * per;
  const long b = (long)HW::block_y();
  u32x4 v = {0u, 0u, 0u, 0u};
  if (r < p.rows) {
    const char* s = (const char*)p.src + (b * p.s_batch + (long)r * p.s_row + c0) * p.esize;
    if (p.esize == 2) {
#pragma unroll
      for (int e = 0; e < 8; e++)
        if (c0 + e < p.cols) v[e >> 1] |= (uint32_t)HW::global_load_u16(s + 2 * e) << (16 * (e & 1));
    } else {
#pragma unroll
      for (int e = 0; e < 4; e++)
        if (c0 + e < p.cols) v[e] = HW::global_load_u32(s + 4 * e);
    }
  }
  HW::global_store16((char*)p.dst + (b * p.d_batch + (long)r * p.d_row + c0) * p.esize, v);
}

// dst[b][r][c] = src[b][r][c] for r < rows, c < cols: the source is a padded image (16-byte
// aligned rows, one 16-byte load per thread), the destination needs element alignment only.
// grid.x covers rows * cols_d * esize / 16 threads.
template <class HW>
__global__ void __launch_bounds__(PACK_THREADS) alcop_unpack(const PackParams p)
{
  const int per = 16 / p.esize, cpr = p.cols_d / per;
  const long idx = (long)HW::block_x() * PACK_THREADS + HW::wave_id() * 64 + HW::lane_id();
  if (idx >= (long)p.rows * cpr) return;
  const int r = (int)(idx / cpr), c0 = (int)(idx - (long)r * cpr) * per;
  if (c0 >= p.cols) return;
  const long b = (long)HW::block_y();
  const char* s = (const char*)p.src + (b * p.s_batch + (long)r * p.s_row + c0) * p.esize;
  const u32x4 v = __builtin_bit_cast(u32x4, HW::global_load_f32x4((const float*)s));
  char* d = (char*)p.dst + (b * p.d_batch + (long)r * p.d_row + c0) * p.esize;
  if (p.esize == 2) {
#pragma unroll
    for (int e = 0; e < 8; e++)
      if (c0 + e < p.cols) HW::global_store_u16(d + 2 * e, (uint16_t)(v[e >> 1] >> (16 * (e & 1))));
  } else {
#pragma unroll
    for (int e = 0; e < 4; e++)
      if (c0 + e < p.cols) HW::global_store_u32(d + 4 * e, v[e]);
  }
}

}  // namespace alcop
