// Split-K variants for GEMM / batched matmul (A stored M x K or K x M; B stored K x N or N x K), and the
// launcher of the reduction step.
#include <mutex>

#include "alcop_instantiate.hip.h"
namespace alcop {

// Scratch memory of the allocation-free split-K entry point: the fp32 partial tiles of one call.
// Every GPU the library runs on holds its own copy of the array, at its own address, until the
// process ends.  In host code the array's name only stands for the symbol: the address a kernel
// can use is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[kSplitkStaticBytes];

hipError_t splitk_scratch(void** ptr, size_t* bytes)
{
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* per_device[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(mu);
  if (per_device[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // with device `dev` current
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    per_device[dev] = p;
  }
  *ptr = per_device[dev];
  *bytes = sizeof(scratch);
  return hipSuccess;
}

void register_splitk_gemm(std::vector<KernelEntry>& t)
{
  ALCOP_SPLITK_PIPES(t, 0, 128, 128, 64, 64, 64, 0, 0)
  ALCOP_SPLITK_PIPES(t, 0, 128, 64, 64, 64, 32, 0, 0)
  ALCOP_SPLITK_PIPES(t, 0, 64, 64, 64, 32, 32, 0, 0)
  ALCOP_SPLITK_PIPES(t, 0, 256, 128, 64, 128, 64, 0, 0)
  ALCOP_SPLITK_PIPES(t, 1, 128, 128, 64, 64, 64, 0, 0)
  ALCOP_SPLITK_PIPES(t, 1, 64, 64, 64, 32, 32, 0, 0)
  ALCOP_SPLITK_PIPES(t, 1, 256, 128, 64, 128, 64, 0, 0)
  ALCOP_SPLITK_PIPES(t, 0, 128, 128, 64, 64, 64, 1, 0)
  ALCOP_SPLITK_PIPES(t, 0, 64, 64, 64, 32, 32, 1, 0)
  ALCOP_SPLITK_PIPES(t, 1, 128, 128, 64, 64, 64, 1, 0)
  // A stored K x M, B stored K x N
  ALCOP_SPLITK_PIPES_TA(t, 0, 128, 128, 64, 64, 64, 0)
  ALCOP_SPLITK_PIPES_TA(t, 0, 64, 64, 64, 32, 32, 0)
  ALCOP_SPLITK_PIPES_TA(t, 1, 128, 128, 64, 64, 64, 0)
  ALCOP_SPLITK_PIPES_TA(t, 1, 64, 64, 64, 32, 32, 0)
}

hipError_t launch_splitk_reduce(const ReduceParams& p, dim3 grid, hipStream_t st)
{
  alcop_splitk_reduce<Gfx950><<<grid, dim3(REDUCE_THREADS), 0, st>>>(p);
  return hipGetLastError();
}
}  // namespace alcop
