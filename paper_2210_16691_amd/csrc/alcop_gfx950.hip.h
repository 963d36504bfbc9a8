// gfx950 (MI355X) implementation of the hardware operations the pipelined main loop is written
// against (the HW template argument of alcop_mainloop).
//
// Facts about the instructions used here, established by probing the hardware:
//   buffer_load_dwordx4 ... lds   writes lane l's 16 bytes at M0 + 16*l; an offset at or beyond the
//                                 descriptor's num_records writes zeros and fetches nothing
//   ds_read_b64_tr_b16            per 16-lane group: lane i receives, as element e, element i%4
//                                 of the 8 bytes addressed by lane 4e + i/4 (four 4x4 transposes)
//   v_mfma_f32_32x32x16_{f16,bf16}  X lane l = row l%32, k = 8*(l/32)..+7; Y likewise by column;
//                                 D lane l = column l%32, rows 8*(v/4) + 4*(l/32) + v%4
// The direct-to-LDS loads and the waits are inline asm on purpose: the compiler treats a builtin
// LDS-DMA as a store to LDS and would drain the vector-memory counter before the next LDS read,
// which serialises the stages.  With asm it sees neither the loads nor their counter; the waits
// are placed by the loop from the stage count (paper Sec. 4.2 step 5).
#pragma once
#include <hip/hip_runtime.h>

#include "alcop_kernel.hip.h"

namespace alcop {

#define ALCOP_LDS __attribute__((address_space(3)))

struct Gfx950 {
  using Rsrc = __amdgpu_buffer_rsrc_t;
  static constexpr bool kSwizzle = true;   // LDS tile images are bank-conflict-free permutations

  // lane within the wavefront, and the wavefront's index within the block (a scalar)
  __device__ static __forceinline__ int lane_id() { return threadIdx.x & 63; }
  __device__ static __forceinline__ int wave_id()
  {
    return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  }
  __device__ static __forceinline__ uint32_t block_x() { return blockIdx.x; }
  __device__ static __forceinline__ uint32_t block_y() { return blockIdx.y; }
  __device__ static __forceinline__ uint32_t block_z() { return blockIdx.z; }

  __device__ static __forceinline__ uint32_t lds_base()
  {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    return (uint32_t)(uintptr_t)(ALCOP_LDS unsigned char*)smem;
  }

  // Buffer resource for a wave-uniform base address.  The words are passed through
  // readfirstlane so that the descriptor provably lives in scalar registers.
  __device__ static __forceinline__ Rsrc make_rsrc(const void* base, int bytes)
  {
    const uint64_t a = (uint64_t)(uintptr_t)base;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    const int n = __builtin_amdgcn_readfirstlane(bytes);
    return __builtin_amdgcn_make_buffer_rsrc((void*)(uintptr_t)(((uint64_t)hi << 32) | lo), 0, n,
                                             0x00020000);
  }

  __device__ static __forceinline__ void dma16(Rsrc rsrc, uint32_t voff, uint32_t lds_dst)
  {
    // M0 holds the wave-uniform LDS destination; lane l lands at M0 + 16*l.
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_dst), "v"(voff), "s"(rsrc)
                 : "memory");
  }

  __device__ static __forceinline__ void touch4(const char* gptr, uint32_t lds_dst)
  {
    // 4-byte direct-to-LDS load per lane into a landing pad nobody reads: its only purpose is
    // to bring the 128-byte line it touches into L2 ahead of the tile loads.
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
                 :
                 : "s"(lds_dst), "v"(gptr)
                 : "memory");
  }

  template <int N>
  __device__ static __forceinline__ void wait_vm()
  {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
  }
  __device__ static __forceinline__ void wait_lds()
  {
    asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");
  }
  __device__ static __forceinline__ void block_barrier() { __builtin_amdgcn_s_barrier(); }
  // nothing may be scheduled across this point
  __device__ static __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

  template <int DT>
  __device__ static __forceinline__ f32x16 mma(u32x4 x, u32x4 y, f32x16 acc)
  {
    if constexpr (DT == 0)
      return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, x),
                                                    __builtin_bit_cast(f16x8, y), acc, 0, 0, 0);
    else
      return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, x),
                                                     __builtin_bit_cast(bf16x8, y), acc, 0, 0, 0);
  }

  __device__ static __forceinline__ u32x4 lds_read16(uint32_t addr)
  {
    return *(const ALCOP_LDS u32x4*)(uintptr_t)addr;
  }
  __device__ static __forceinline__ u32x2 lds_read_tr8(uint32_t addr)
  {
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ALCOP_LDS s16x4*)(uintptr_t)addr);
    return __builtin_bit_cast(u32x2, v);
  }
  template <class V>
  __device__ static __forceinline__ void lds_write(uint32_t addr, V v)
  {
    *(ALCOP_LDS V*)(uintptr_t)addr = v;
  }

  // 16-byte store that bypasses the caches' retention (C is written once and not re-read)
  __device__ static __forceinline__ void global_store16(void* ptr, u32x4 v)
  {
    __builtin_nontemporal_store(v, (u32x4*)ptr);
  }
  __device__ static __forceinline__ f32x4 global_load_f32x4(const float* ptr)
  {
    return *(const f32x4*)ptr;
  }
  // element-wise accesses of the pack / unpack kernels (any element-aligned address)
  __device__ static __forceinline__ uint16_t global_load_u16(const void* ptr) { return *(const uint16_t*)ptr; }
  __device__ static __forceinline__ uint32_t global_load_u32(const void* ptr) { return *(const uint32_t*)ptr; }
  __device__ static __forceinline__ void global_store_u16(void* ptr, uint16_t v) { *(uint16_t*)ptr = v; }
  __device__ static __forceinline__ void global_store_u32(void* ptr, uint32_t v) { *(uint32_t*)ptr = v; }
  // fp32 -> output element, round to nearest even
  template <class OT>
  __device__ static __forceinline__ OT cvt(float v)
  {
    return (OT)v;
  }
};

}  // namespace alcop
