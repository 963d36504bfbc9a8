// Table of the kernels built into the library: one entry per template instance.
#pragma once
#include <hip/hip_runtime.h>
#include <vector>

#include "alcop_kernel.hip.h"

namespace alcop {

struct KernelEntry {
  int dt, bm, bn, bk, wm, wn, stages, reg_stages, fuse, bl, am, al;
  int lds_bytes, threads, loads_per_stage;
  hipError_t (*launch)(const Params&, dim3, hipStream_t);
};

// Sub-tables, one per source shard (compiled in parallel).
void register_f16_kn_big(std::vector<KernelEntry>&);
void register_f16_kn_mid(std::vector<KernelEntry>&);
void register_f16_kn_small(std::vector<KernelEntry>&);
void register_bf16_kn(std::vector<KernelEntry>&);
void register_nk(std::vector<KernelEntry>&);
void register_conv(std::vector<KernelEntry>&);
void register_ta(std::vector<KernelEntry>&);

const std::vector<KernelEntry>& registry();

}  // namespace alcop
