// Table of the kernels built into the library: one entry per template instance.
#pragma once
#include <hip/hip_runtime.h>
#include <vector>

#include "alcop_kernel.hip.h"
#include "alcop_pack.hip.h"
#include "alcop_splitk.hip.h"

namespace alcop {

struct KernelEntry {
  int dt, bm, bn, bk, wm, wn, stages, reg_stages, fuse, bl, am, al;
  int sk;   // 1: split-K variant (grid.z slices of the reduction axis, fp32 partial tiles)
  int pf;   // 1: the kernel has the HBM -> L2 touch level (schedules with l2_prefetch > 0)
  int st;   // 1: persistent producer / consumer kernel (schedule variant 2)
  int lds_bytes, threads, loads_per_stage;
  int patch_off;   // am == 3: LDS offset of the input patch (its size is per call)
  hipError_t (*launch)(const Params&, dim3, hipStream_t);
  // what the first launch would do besides launching (the opt-in to the kernel's LDS size), so
  // that alcop_init can do it ahead of time; may be null
  hipError_t (*prepare)() = nullptr;
};

// Sub-tables, one per source shard (compiled in parallel).
void register_f16_kn_big(std::vector<KernelEntry>&);
void register_f16_kn_mid(std::vector<KernelEntry>&);
void register_f16_kn_small(std::vector<KernelEntry>&);
void register_bf16_kn(std::vector<KernelEntry>&);
void register_nk(std::vector<KernelEntry>&);
void register_conv(std::vector<KernelEntry>&);
void register_ta(std::vector<KernelEntry>&);
void register_conv_krsc(std::vector<KernelEntry>&);
void register_conv_anyc(std::vector<KernelEntry>&);
void register_conv_patch(std::vector<KernelEntry>&);
void register_bk128(std::vector<KernelEntry>&);
void register_deep(std::vector<KernelEntry>&);
void register_wide(std::vector<KernelEntry>&);
void register_pf(std::vector<KernelEntry>&);
void register_stream(std::vector<KernelEntry>&);
void register_splitk_gemm(std::vector<KernelEntry>&);
void register_splitk_conv(std::vector<KernelEntry>&);

// Second step of a split-K product (alcop_splitk.hip.h).
hipError_t launch_splitk_reduce(const ReduceParams& p, dim3 grid, hipStream_t st);

// Copies into and out of the padded workspace images (alcop_pack.hip.h); grid.y = batch entries.
hipError_t launch_pack(const PackParams& p, int batch, hipStream_t st);
hipError_t launch_unpack(const PackParams& p, int batch, hipStream_t st);

// Device address and size of the library's own scratch array on the current device (set up on
// the first call per device; allocates nothing afterwards).  Its size is part of the interface
// (ALCOP_SPLITK_STATIC_BYTES in alcop.h; alcop_api.cpp checks that the two agree).
constexpr size_t kSplitkStaticBytes = 32u << 20;
hipError_t splitk_scratch(void** ptr, size_t* bytes);

const std::vector<KernelEntry>& registry();

}  // namespace alcop
