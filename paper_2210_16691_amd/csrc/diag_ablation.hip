// libalcop_diag.so: the product's kernel template instantiated with hardware-policy classes that
// leave out one class of operation each, to measure what the others cost and how well loads and
// compute overlap (see include/alcop_diag.h).  An ablated kernel computes garbage; it performs a
// subset of the full kernel's memory accesses, at the same addresses, with the same launch shape.
#include <cstring>

#include "../../include/alcop_diag.h"
#include "alcop_gfx950.hip.h"
#include "alcop_stream.hip.h"

namespace alcop {
namespace {

template <int DROP>
struct Ablated : Gfx950 {
  static constexpr bool kSwizzle = !(DROP & ALCOP_DIAG_NO_SWIZZLE);
  __device__ static __forceinline__ void dma16(Rsrc rsrc, uint32_t voff, uint32_t lds_dst)
  {
    if constexpr (!(DROP & ALCOP_DIAG_NO_DMA)) Gfx950::dma16(rsrc, voff, lds_dst);
  }
  __device__ static __forceinline__ void touch4(const char* gptr, uint32_t lds_dst)
  {
    if constexpr (!(DROP & ALCOP_DIAG_NO_DMA)) Gfx950::touch4(gptr, lds_dst);
  }
  __device__ static __forceinline__ u32x4 lds_read16(uint32_t addr)
  {
    if constexpr (DROP & ALCOP_DIAG_NO_LDS_READ) {
      u32x4 v;
      asm volatile("" : "=v"(v) : "v"(addr));   // registers as they are: no instruction
      return v;
    } else {
      return Gfx950::lds_read16(addr);
    }
  }
  __device__ static __forceinline__ u32x2 lds_read_tr8(uint32_t addr)
  {
    if constexpr (DROP & ALCOP_DIAG_NO_LDS_READ) {
      u32x2 v;
      asm volatile("" : "=v"(v) : "v"(addr));
      return v;
    } else {
      return Gfx950::lds_read_tr8(addr);
    }
  }
  template <int DT>
  __device__ static __forceinline__ f32x16 mma(u32x4 x, u32x4 y, f32x16 acc)
  {
    if constexpr (DROP & ALCOP_DIAG_NO_MFMA) {
      asm volatile("" : : "v"(x), "v"(y));      // keeps the fragment reads alive
      return acc;
    } else {
      return Gfx950::mma<DT>(x, y, acc);
    }
  }
  __device__ static __forceinline__ void block_barrier()
  {
    if constexpr (!(DROP & ALCOP_DIAG_NO_BARRIER)) Gfx950::block_barrier();
  }
  __device__ static __forceinline__ void global_store16(void* ptr, u32x4 v)
  {
    if constexpr (DROP & ALCOP_DIAG_NO_STORE)
      asm volatile("" : : "v"(ptr), "v"(v));    // the conversions and the staging stay
    else
      Gfx950::global_store16(ptr, v);
  }
};

struct Config {
  const char* name;
  int dt, bm, bn, bk;
  hipError_t (*launch)(int drop, const Params& p, dim3 grid);
  int persistent;   // 1: producer / consumer kernel, launched with one block per compute unit at most
};

template <class C, int DROP>
hipError_t launch_one(const Params& p, dim3 grid)
{
  static bool attr = false;   // single-threaded measurement tool
  if (!attr) {
    hipError_t e = hipFuncSetAttribute((const void*)alcop_mainloop<C, Ablated<DROP>>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr = true;
  }
  alcop_mainloop<C, Ablated<DROP>><<<grid, dim3(C::NT), C::LDS_BYTES, 0>>>(p);
  return hipGetLastError();
}

template <class C, int DROP>
hipError_t launch_one_stream(const Params& p, dim3 grid)
{
  static bool attr = false;   // single-threaded measurement tool
  if (!attr) {
    hipError_t e = hipFuncSetAttribute((const void*)alcop_stream<C, Ablated<DROP>>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr = true;
  }
  alcop_stream<C, Ablated<DROP>><<<grid, dim3(C::NT), C::LDS_BYTES, 0>>>(p);
  return hipGetLastError();
}

template <class C>
hipError_t launch_cfg_stream(int drop, const Params& p, dim3 grid)
{
  switch (drop) {
    case 0: return launch_one_stream<C, 0>(p, grid);
    case 1: return launch_one_stream<C, 1>(p, grid);
    case 2: return launch_one_stream<C, 2>(p, grid);
    case 4: return launch_one_stream<C, 4>(p, grid);
    case 8: return launch_one_stream<C, 8>(p, grid);
    case 3: return launch_one_stream<C, 3>(p, grid);
    case 6: return launch_one_stream<C, 6>(p, grid);
    case 7: return launch_one_stream<C, 7>(p, grid);
    case 16: return launch_one_stream<C, 16>(p, grid);
    case 23: return launch_one_stream<C, 23>(p, grid);
    case 32: return launch_one_stream<C, 32>(p, grid);
    case 64: return launch_one_stream<C, 64>(p, grid);
    default: return hipErrorInvalidValue;
  }
}

template <class C>
hipError_t launch_cfg(int drop, const Params& p, dim3 grid)
{
  switch (drop) {
    case 0: return launch_one<C, 0>(p, grid);
    case 1: return launch_one<C, 1>(p, grid);
    case 2: return launch_one<C, 2>(p, grid);
    case 4: return launch_one<C, 4>(p, grid);
    case 8: return launch_one<C, 8>(p, grid);
    case 3: return launch_one<C, 3>(p, grid);
    case 6: return launch_one<C, 6>(p, grid);
    case 7: return launch_one<C, 7>(p, grid);
    case 16: return launch_one<C, 16>(p, grid);
    case 23: return launch_one<C, 23>(p, grid);
    case 32: return launch_one<C, 32>(p, grid);
    case 64: return launch_one<C, 64>(p, grid);
    default: return hipErrorInvalidValue;
  }
}

// a kernel that does nothing: what a launch costs when launches follow each other on one stream
__global__ void empty_kernel() {}

const Config kConfigs[] = {
    {"f16 128x128x64 w64x64 S4 R2 F1", 0, 128, 128, 64, &launch_cfg<KCfg<0, 128, 128, 64, 64, 64, 4, 2, 1, 0, 0>>},
    {"f16 128x128x64 w64x64 S3 R4 F1", 0, 128, 128, 64, &launch_cfg<KCfg<0, 128, 128, 64, 64, 64, 3, 4, 1, 0, 0>>},
    {"f16 128x128x64 w64x64 S1 R1 F0", 0, 128, 128, 64, &launch_cfg<KCfg<0, 128, 128, 64, 64, 64, 1, 1, 0, 0, 0>>},
    {"bf16 256x256x32 w128x64 S3 R2 F1", 1, 256, 256, 32, &launch_cfg<KCfg<1, 256, 256, 32, 128, 64, 3, 2, 1, 0, 0>>},
    {"bf16 256x256x32 w128x64 S1 R1 F0", 1, 256, 256, 32, &launch_cfg<KCfg<1, 256, 256, 32, 128, 64, 1, 1, 0, 0, 0>>},
    {"f16 128x128x64 w64x64 S3 persistent F0", 0, 128, 128, 64,
     &launch_cfg_stream<SCfg<0, 128, 128, 64, 64, 64, 3, 0, 0, 0, 0>>, 1},
    {"f16 128x128x64 w64x64 S3 persistent F1", 0, 128, 128, 64,
     &launch_cfg_stream<SCfg<0, 128, 128, 64, 64, 64, 3, 0, 0, 0, 1>>, 1},
};
constexpr int kNumConfigs = (int)(sizeof(kConfigs) / sizeof(kConfigs[0]));

}  // namespace
}  // namespace alcop

extern "C" {

int alcop_diag_configs(void) { return alcop::kNumConfigs; }

const char* alcop_diag_config_name(int i)
{
  return (i >= 0 && i < alcop::kNumConfigs) ? alcop::kConfigs[i].name : nullptr;
}

int alcop_diag_time(int config, int drop, const void* A, const void* B, void* C, int M, int N,
                    int K, int iters, double* mean_us)
{
  using namespace alcop;
  if (config < 0 || config >= kNumConfigs || !A || !B || !C || !mean_us || iters <= 0) return -1;
  const Config& cf = kConfigs[config];
  if (M <= 0 || N <= 0 || K <= 0 || M % cf.bm || N % cf.bn || K % cf.bk) return -1;
  if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) & 15) return -1;
  if ((double)M * K * 2 >= 2147483648.0 || (double)K * N * 2 >= 2147483648.0) return -1;
  if (drop != 0 && drop != 1 && drop != 2 && drop != 4 && drop != 8 && drop != 3 && drop != 6 && drop != 7 &&
      drop != 16 && drop != 23 && drop != 32 && drop != 64)
    return -1;
  Params p;
  std::memset(&p, 0, sizeof(p));
  p.A = A;
  p.B = B;
  p.C = C;
  p.M = M;
  p.N = N;
  p.K = K;
  p.lda = K;
  p.ldb = N;
  p.ldc = N;
  p.out_dtype = cf.dt;
  p.ntm = M / cf.bm;
  p.ntn = N / cf.bn;
  p.raster = 1;
  p.group_m = p.ntm < 8 ? p.ntm : 8;
  p.alpha = 1.0f;
  p.pf_pa = p.pf_pb = 1;
  dim3 grid((unsigned)(p.ntm * p.ntn), 1, 1);
  if (cf.persistent) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      return -2;
    p.sbatch = 1;
    p.sgrid = p.ntm * p.ntn < cus ? p.ntm * p.ntn : cus;
    grid = dim3((unsigned)p.sgrid, 1, 1);
  }
  for (int i = 0; i < 20; i++)
    if (cf.launch(drop, p, grid) != hipSuccess) return -2;
  if (hipDeviceSynchronize() != hipSuccess) return -2;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -2;
  double best = 1e30;
  int rc = 0;
  for (int rep = 0; rep < 3 && rc == 0; rep++) {
    if (hipEventRecord(e0, 0) != hipSuccess) rc = -2;
    for (int i = 0; i < iters && rc == 0; i++)
      if (cf.launch(drop, p, grid) != hipSuccess) rc = -2;
    if (rc == 0 && (hipEventRecord(e1, 0) != hipSuccess || hipEventSynchronize(e1) != hipSuccess)) rc = -2;
    float ms = 0;
    if (rc == 0 && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = -2;
    if (rc == 0 && ms * 1e3 / iters < best) best = ms * 1e3 / iters;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc) return rc;
  *mean_us = best;
  return 0;
}

int alcop_diag_launch_floor(int blocks, int threads, int iters, double* mean_us)
{
  if (blocks <= 0 || blocks > 65536 || threads <= 0 || threads > 1024 || iters <= 0 || !mean_us) return -1;
  for (int i = 0; i < 20; i++) alcop::empty_kernel<<<dim3((unsigned)blocks), dim3((unsigned)threads), 0, 0>>>();
  if (hipDeviceSynchronize() != hipSuccess) return -2;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -2;
  double best = 1e30;
  int rc = 0;
  for (int rep = 0; rep < 3 && rc == 0; rep++) {
    if (hipEventRecord(e0, 0) != hipSuccess) rc = -2;
    for (int i = 0; i < iters; i++) alcop::empty_kernel<<<dim3((unsigned)blocks), dim3((unsigned)threads), 0, 0>>>();
    if (rc == 0 && (hipGetLastError() != hipSuccess || hipEventRecord(e1, 0) != hipSuccess ||
                    hipEventSynchronize(e1) != hipSuccess))
      rc = -2;
    float ms = 0;
    if (rc == 0 && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = -2;
    if (rc == 0 && ms * 1e3 / iters < best) best = ms * 1e3 / iters;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc) return rc;
  *mean_us = best;
  return 0;
}

}  // extern "C"
