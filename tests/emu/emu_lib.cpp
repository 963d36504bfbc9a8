// CPU build of the library for tests: the product's host code (alcop_api.cpp, alcop_model.cpp,
// compiled unchanged) linked with a kernel table whose launchers run the kernel template on the
// functional hardware model of emu_hw.h instead of launching it on a GPU.  Operands are host
// memory.  Only a sample of the product's instances is built (each costs compile time); the
// sample covers both element types, every operand layout, the convolution gather, 4- and
// 8-wave blocks, one to four stages, single- and multi-level, fused and unfused.
#include <hip/hip_runtime.h>

#include "emu_hw.h"
#include "alcop_registry.h"

namespace alcop {

template <class C>
hipError_t launch_emulated(const Params& p, dim3 grid, hipStream_t)
{
  emu::run_grid(&emu::mainloop_entry<C>, &p, C::NT, dynamic_lds_bytes<C>(p), grid.x, grid.y, grid.z);
  return hipSuccess;
}

template <int DT, int BM, int BN, int BK, int WM, int WN, int S, int R, int F, int BL, int AM,
          int AL = 0, int SK = 0, int PF = 0>
void add(std::vector<KernelEntry>& t)
{
  using C = KCfg<DT, BM, BN, BK, WM, WN, S, R, F, BL, AM, AL, SK, PF>;
  t.push_back(KernelEntry{DT, BM, BN, BK, WM, WN, S, R, F, BL, AM, AL, SK, PF, 0, C::LDS_BYTES, C::NT, C::L,
                          C::PATCH_OFF, &launch_emulated<C>});
}

template <class C>
hipError_t launch_emulated_stream(const Params& p, dim3 grid, hipStream_t)
{
  emu::run_grid(&emu::stream_entry<C>, &p, C::NT, C::LDS_BYTES, grid.x, grid.y, grid.z);
  return hipSuccess;
}

template <int DT, int BM, int BN, int BK, int WM, int WN, int S, int BL, int AM, int AL = 0, int FU = 1>
void add_stream(std::vector<KernelEntry>& t)
{
  using C = SCfg<DT, BM, BN, BK, WM, WN, S, BL, AM, AL, FU>;
  t.push_back(KernelEntry{DT, BM, BN, BK, WM, WN, S, FU == 2 ? 4 : 2, FU ? 1 : 0, BL, AM, AL, 0, 0, 1, C::LDS_BYTES, C::NT, C::L, 0,
                          &launch_emulated_stream<C>});
}

#if EMU_PART == 0
void emu_part_0(std::vector<KernelEntry>& t)
{
  // every pipelining variant of one tile
  add<0, 128, 128, 64, 64, 64, 1, 1, 0, 0, 0>(t);
  add<0, 128, 128, 64, 64, 64, 2, 1, 0, 0, 0>(t);
  add<0, 128, 128, 64, 64, 64, 3, 1, 0, 0, 0>(t);
  add<0, 128, 128, 64, 64, 64, 1, 2, 0, 0, 0>(t);
  add<0, 128, 128, 64, 64, 64, 2, 2, 0, 0, 0>(t);
  add<0, 128, 128, 64, 64, 64, 4, 2, 0, 0, 0>(t);
  add<0, 128, 128, 64, 64, 64, 2, 2, 1, 0, 0>(t);
  add<0, 128, 128, 64, 64, 64, 3, 2, 1, 0, 0>(t);
  add<0, 128, 128, 64, 64, 64, 4, 2, 1, 0, 0>(t);
  add<0, 128, 128, 32, 64, 64, 3, 2, 1, 0, 0>(t);
  // with the HBM -> L2 touch level
  add<0, 128, 128, 64, 64, 64, 4, 2, 1, 0, 0, 0, 0, 1>(t);
  add<0, 128, 128, 64, 64, 64, 4, 2, 1, 1, 0, 0, 0, 1>(t);
  add<0, 64, 64, 32, 32, 32, 4, 2, 1, 0, 0, 0, 0, 1>(t);
  add<0, 128, 128, 64, 64, 64, 3, 4, 1, 0, 0, 0, 0, 1>(t);
  add<1, 128, 128, 64, 64, 64, 3, 2, 1, 0, 0, 1, 0, 1>(t);   // A stored K x M
}
#elif EMU_PART == 1
void emu_part_1(std::vector<KernelEntry>& t)
{
  add<0, 256, 256, 32, 128, 64, 2, 2, 1, 0, 0>(t);     // 8 waves
  add<0, 256, 128, 64, 128, 64, 2, 2, 1, 0, 0>(t);
  add<0, 64, 64, 32, 32, 32, 1, 1, 0, 0, 0>(t);
  add<0, 64, 64, 32, 32, 32, 4, 2, 1, 0, 0>(t);
  add<0, 64, 64, 64, 32, 32, 3, 2, 1, 0, 0>(t);
  add<0, 256, 64, 64, 64, 64, 3, 1, 0, 0, 0>(t);
  add<0, 64, 128, 64, 32, 64, 3, 2, 1, 0, 0>(t);
  add<1, 128, 128, 64, 64, 64, 3, 2, 1, 0, 0>(t);      // bf16
  add<1, 64, 64, 32, 32, 32, 2, 1, 0, 0, 0>(t);
  add<0, 128, 128, 128, 64, 64, 2, 2, 1, 0, 0>(t);     // k-tile of 128
  add<0, 128, 128, 128, 64, 64, 1, 1, 0, 0, 0>(t);
  add<0, 64, 64, 128, 32, 32, 4, 2, 1, 0, 0>(t);
  add<0, 64, 64, 128, 32, 32, 4, 2, 1, 0, 0, 0, 0, 1>(t);   // ... with L2 touches
  add<0, 128, 64, 128, 64, 32, 2, 1, 0, 0, 0>(t);
  add<1, 128, 128, 128, 64, 64, 2, 2, 0, 1, 0>(t);     // ... B stored N x K, bf16
  add<0, 64, 64, 128, 32, 32, 3, 2, 1, 1, 0>(t);
}
#elif EMU_PART == 2
void emu_part_2(std::vector<KernelEntry>& t)
{
  add<0, 128, 128, 64, 64, 64, 1, 1, 0, 1, 0>(t);      // B stored N x K
  add<0, 128, 128, 64, 64, 64, 2, 2, 0, 1, 0>(t);
  add<0, 128, 128, 64, 64, 64, 4, 2, 1, 1, 0>(t);
  add<0, 128, 128, 32, 64, 64, 3, 2, 1, 1, 0>(t);
  add<0, 64, 64, 64, 32, 32, 3, 2, 1, 1, 0>(t);
  add<1, 64, 64, 32, 32, 32, 3, 2, 1, 1, 0>(t);
  add<0, 128, 128, 64, 64, 64, 3, 2, 1, 0, 0, 1>(t);   // A stored K x M
  add<0, 128, 128, 64, 64, 64, 2, 1, 0, 0, 0, 1>(t);
  add<0, 64, 64, 32, 32, 32, 4, 2, 1, 0, 0, 1>(t);
  add<0, 128, 128, 64, 64, 64, 3, 2, 1, 1, 0, 1>(t);   // A stored K x M, B stored N x K
  add<1, 64, 64, 32, 32, 32, 2, 2, 1, 1, 0, 1>(t);
}
#elif EMU_PART == 4
void emu_part_4(std::vector<KernelEntry>& t)
{
  // split-K variants
  add<0, 128, 128, 64, 64, 64, 1, 1, 0, 0, 0, 0, 1>(t);
  add<0, 128, 128, 64, 64, 64, 3, 2, 1, 0, 0, 0, 1>(t);
  add<0, 64, 64, 64, 32, 32, 4, 2, 1, 0, 0, 0, 1>(t);
  add<1, 128, 128, 64, 64, 64, 2, 2, 1, 0, 0, 0, 1>(t);
  add<0, 128, 128, 64, 64, 64, 3, 2, 1, 1, 0, 0, 1>(t);   // B stored N x K
  add<0, 64, 64, 64, 32, 32, 2, 2, 1, 1, 0, 0, 1>(t);
  add<0, 128, 64, 64, 64, 32, 3, 2, 1, 0, 1, 0, 1>(t);    // convolution
  add<0, 64, 64, 64, 32, 32, 1, 1, 0, 0, 1, 0, 1>(t);
  add<0, 64, 128, 64, 32, 64, 4, 2, 1, 0, 1, 0, 1>(t);
  add<0, 128, 128, 64, 64, 64, 3, 2, 1, 0, 0, 1, 1>(t);   // A stored K x M
  add<1, 64, 64, 64, 32, 32, 2, 2, 1, 0, 0, 1, 1>(t);
}
#elif EMU_PART == 5
void emu_part_5(std::vector<KernelEntry>& t)
{
  // register pipelines deeper than two stages (fused only)
  add<0, 128, 128, 64, 64, 64, 4, 4, 1, 0, 0>(t);      // D = 3 of 4 fragments: synchronisation in step 1
  add<0, 128, 128, 64, 64, 64, 2, 3, 1, 0, 0>(t);      // R = 3 with 4 fragments: body of three periods
  add<0, 128, 128, 32, 64, 64, 3, 3, 1, 0, 0>(t);      // D = all fragments of a k-tile
  add<0, 64, 64, 64, 32, 32, 3, 4, 1, 0, 0>(t);
  add<0, 256, 256, 32, 128, 64, 2, 3, 1, 0, 0>(t);     // 8 waves
  add<0, 128, 128, 128, 64, 64, 2, 4, 1, 0, 0>(t);     // k-tile of 128: 8 fragments
  add<1, 128, 128, 64, 64, 64, 3, 4, 1, 0, 0>(t);      // bf16
  add<0, 128, 128, 64, 64, 64, 4, 4, 1, 1, 0>(t);      // B stored N x K
  add<1, 64, 64, 32, 32, 32, 4, 3, 1, 1, 0>(t);
  add<0, 128, 128, 64, 64, 64, 3, 4, 1, 0, 0, 1>(t);   // A stored K x M
  add<0, 128, 128, 64, 64, 64, 3, 3, 1, 1, 0, 1>(t);
  add<0, 128, 64, 64, 64, 32, 3, 4, 1, 0, 1>(t);       // convolution gather
  add<0, 128, 64, 32, 64, 32, 4, 3, 1, 0, 2>(t);
  add<0, 128, 64, 64, 64, 32, 3, 4, 1, 1, 1>(t);       // KRSC weights
  add<0, 256, 64, 64, 64, 64, 3, 4, 1, 0, 3>(t);       // input patch resident in LDS
  add<0, 128, 128, 64, 64, 64, 3, 4, 1, 0, 0, 0, 1>(t);   // split-K
}
#elif EMU_PART == 6
void emu_part_6(std::vector<KernelEntry>& t)
{
  // persistent producer / consumer kernels (schedule variant 2)
  add_stream<0, 128, 128, 64, 64, 64, 3, 0, 0>(t);
  add_stream<0, 128, 128, 64, 64, 64, 2, 1, 0>(t);     // B stored N x K
  add_stream<0, 128, 64, 32, 64, 32, 4, 0, 0>(t);
  add_stream<0, 64, 64, 64, 32, 32, 3, 1, 0>(t);
  add_stream<1, 64, 64, 32, 32, 32, 2, 0, 0>(t);       // bf16
  add_stream<0, 256, 64, 64, 64, 64, 2, 0, 0>(t);
  add_stream<0, 128, 64, 64, 64, 32, 3, 0, 1>(t);      // convolution gather
  add_stream<0, 64, 64, 32, 32, 32, 4, 0, 1>(t);
  add_stream<0, 256, 64, 64, 64, 64, 2, 0, 1>(t);
  // ... with the deep register pipeline (three fragments in flight, the barrier early in the k-tile)
  add_stream<0, 128, 128, 64, 64, 64, 3, 0, 0, 0, 2>(t);
  add_stream<0, 128, 128, 64, 64, 64, 2, 1, 0, 0, 2>(t);
  add_stream<1, 64, 64, 64, 32, 32, 2, 0, 0, 0, 2>(t);
  add_stream<0, 128, 64, 64, 64, 32, 3, 0, 1, 0, 2>(t);
  add_stream<0, 64, 64, 128, 32, 32, 2, 0, 0, 0, 2>(t);      // eight fragments per k-tile
  // ... with the register pipeline restarted in every k-tile
  add_stream<0, 128, 128, 64, 64, 64, 3, 0, 0, 0, 0>(t);
  add_stream<0, 64, 64, 64, 32, 32, 3, 1, 0, 0, 0>(t);
  add_stream<0, 128, 64, 64, 64, 32, 3, 0, 1, 0, 0>(t);
}
#elif EMU_PART == 7
void emu_part_7(std::vector<KernelEntry>& t)
{
  // tiles 192 wide along a contiguous m / n axis: three 64-column LDS images
  add<0, 256, 192, 32, 128, 96, 3, 2, 1, 0, 0>(t);
  add<0, 256, 192, 32, 128, 96, 1, 1, 0, 0, 0>(t);
  add<1, 256, 192, 32, 128, 96, 4, 2, 1, 0, 0>(t);     // bf16
  add<0, 256, 192, 64, 64, 96, 2, 2, 1, 0, 0>(t);      // 8 waves, k-tile of 64
  add<0, 256, 192, 32, 128, 96, 3, 3, 1, 0, 0>(t);     // deep register pipeline
  add<0, 192, 256, 32, 96, 128, 3, 2, 1, 0, 0, 1>(t);  // A stored K x M, 192 rows of C per tile
  add<0, 256, 192, 32, 128, 96, 2, 2, 1, 1, 0>(t);     // B stored N x K: plain rows, 192 of them
  add_stream<0, 128, 192, 32, 64, 96, 3, 0, 0>(t);     // persistent kernels
  add_stream<1, 128, 192, 32, 64, 96, 4, 0, 0, 0, 0>(t);
}
#elif EMU_PART == 3
void emu_part_3(std::vector<KernelEntry>& t)
{
  add<0, 128, 64, 64, 64, 32, 1, 1, 0, 0, 1>(t);       // convolution gather
  add<0, 128, 64, 64, 64, 32, 2, 2, 0, 0, 1>(t);
  add<0, 128, 64, 64, 64, 32, 3, 2, 1, 0, 1>(t);
  add<0, 128, 64, 32, 64, 32, 4, 2, 1, 0, 1>(t);
  add<0, 64, 64, 32, 32, 32, 3, 2, 1, 0, 1>(t);
  add<0, 256, 64, 64, 64, 64, 1, 2, 0, 0, 1>(t);
  add<0, 64, 128, 64, 32, 64, 3, 2, 1, 0, 1>(t);
  add<1, 128, 64, 64, 64, 32, 3, 2, 1, 0, 1>(t);
  add<0, 128, 64, 64, 64, 32, 3, 2, 1, 1, 1>(t);       // KRSC weights
  add<0, 64, 64, 32, 32, 32, 1, 1, 0, 1, 1>(t);
  add<0, 128, 128, 64, 64, 64, 4, 2, 1, 1, 1>(t);
  add<0, 128, 64, 64, 64, 32, 3, 2, 1, 0, 2>(t);       // gather for any channel count (x8)
  add<0, 128, 64, 32, 64, 32, 2, 1, 0, 0, 2>(t);
  add<0, 64, 64, 32, 32, 32, 4, 2, 1, 0, 2>(t);
  add<0, 64, 64, 64, 32, 32, 1, 1, 0, 0, 2>(t);
  add<0, 64, 64, 32, 32, 32, 3, 2, 1, 1, 2>(t);        // ... with KRSC weights
  add<0, 256, 64, 64, 64, 64, 3, 2, 1, 0, 3>(t);       // input patch resident in LDS
  add<0, 256, 64, 64, 64, 64, 1, 1, 0, 0, 3>(t);
  add<0, 128, 64, 64, 64, 32, 2, 2, 0, 0, 3>(t);
  add<0, 128, 64, 32, 64, 32, 4, 2, 1, 0, 3>(t);
  add<0, 64, 64, 32, 32, 32, 2, 1, 0, 0, 3>(t);
  add<1, 128, 64, 64, 64, 32, 3, 2, 1, 0, 3>(t);
}
#else
// the part that is compiled once: the product's sub-table hooks and the test controls
void emu_part_0(std::vector<KernelEntry>&);
void emu_part_1(std::vector<KernelEntry>&);
void emu_part_2(std::vector<KernelEntry>&);
void emu_part_3(std::vector<KernelEntry>&);
void emu_part_4(std::vector<KernelEntry>&);
void emu_part_5(std::vector<KernelEntry>&);
void emu_part_6(std::vector<KernelEntry>&);
void emu_part_7(std::vector<KernelEntry>&);
void register_f16_kn_mid(std::vector<KernelEntry>& t)
{
  emu_part_0(t);
  emu_part_1(t);
  emu_part_2(t);
  emu_part_3(t);
  emu_part_4(t);
  emu_part_5(t);
  emu_part_6(t);
  emu_part_7(t);
}
void register_splitk_gemm(std::vector<KernelEntry>&) {}
void register_splitk_conv(std::vector<KernelEntry>&) {}
void register_conv_krsc(std::vector<KernelEntry>&) {}
void register_conv_anyc(std::vector<KernelEntry>&) {}
void register_conv_patch(std::vector<KernelEntry>&) {}
void register_bk128(std::vector<KernelEntry>&) {}
void register_deep(std::vector<KernelEntry>&) {}
void register_wide(std::vector<KernelEntry>&) {}
void register_pf(std::vector<KernelEntry>&) {}
void register_stream(std::vector<KernelEntry>&) {}

static void reduce_entry(const void* p)
{
  alcop_splitk_reduce<emu::Emu>(*(const ReduceParams*)p);
}
hipError_t launch_splitk_reduce(const ReduceParams& p, dim3 grid, hipStream_t)
{
  emu::run_grid(&reduce_entry, &p, REDUCE_THREADS, 0, grid.x, grid.y, grid.z);
  return hipSuccess;
}
static void pack_entry(const void* p) { alcop_pack<emu::Emu>(*(const PackParams*)p); }
static void unpack_entry(const void* p) { alcop_unpack<emu::Emu>(*(const PackParams*)p); }
hipError_t launch_pack(const PackParams& p, int batch, hipStream_t)
{
  const long threads = (long)p.rows_d * (p.cols_d / (16 / p.esize));
  emu::run_grid(&pack_entry, &p, PACK_THREADS, 0, (unsigned)((threads + PACK_THREADS - 1) / PACK_THREADS),
                (unsigned)batch, 1);
  return hipSuccess;
}
hipError_t launch_unpack(const PackParams& p, int batch, hipStream_t)
{
  const long threads = (long)p.rows * (p.cols_d / (16 / p.esize));
  emu::run_grid(&unpack_entry, &p, PACK_THREADS, 0, (unsigned)((threads + PACK_THREADS - 1) / PACK_THREADS),
                (unsigned)batch, 1);
  return hipSuccess;
}
// host stand-in for the library's device scratch array
hipError_t splitk_scratch(void** ptr, size_t* bytes)
{
  static std::vector<unsigned char> mem(kSplitkStaticBytes);
  *ptr = mem.data();
  *bytes = mem.size();
  return hipSuccess;
}
void register_f16_kn_big(std::vector<KernelEntry>&) {}
void register_f16_kn_small(std::vector<KernelEntry>&) {}
void register_bf16_kn(std::vector<KernelEntry>&) {}
void register_nk(std::vector<KernelEntry>&) {}
void register_conv(std::vector<KernelEntry>&) {}
void register_ta(std::vector<KernelEntry>&) {}
#endif

}  // namespace alcop

#if EMU_PART < 0
extern "C" {

// Forget all registered buffers and logged errors; choose the timing policy of the next runs:
// late_landing != 0: direct-to-LDS data arrives only when a wait forces it (else at issue);
// last_wave_first != 0: the scheduler lets the last wave of a block run ahead (else the first).
void emu_reset(int late_landing, int last_wave_first)
{
  emu::Config& c = emu::cfg();
  c.buffers.clear();
  c.errors.clear();
  c.n_errors = 0;
  c.any_address = false;
  c.late_landing = late_landing != 0;
  c.last_wave_first = last_wave_first != 0;
}

// Declares [ptr, ptr + bytes) as memory the kernel may read (and write, if writable != 0).
void emu_register_buffer(const void* ptr, size_t bytes, int writable)
{
  emu::cfg().buffers.push_back(emu::Buffer{(const char*)ptr, bytes, writable != 0});
}

// Plants a mistake in the model's synchronisation, to show that the checks notice it:
// 1 = every vmcnt wait lets two more loads stay in flight than asked (one more would be
// harmless: the last load of every stage is the L2 touch, which nobody reads); 2 = the block
// barrier does not wait; 3 = vmcnt waits are ignored (loads land only at the final wait);
// 4 = lgkmcnt waits are ignored (LDS reads stay in flight).
void emu_set_mutation(int m) { emu::cfg().mutation = m; }

// any != 0: global accesses are not checked against declared operands (for running code that
// does not declare them); LDS, uniformity and synchronisation checks stay on.
void emu_allow_any_address(int any) { emu::cfg().any_address = any != 0; }

long emu_error_count(void) { return emu::cfg().n_errors; }

// Copies the logged error messages (newline separated, at most cap - 1 characters) into out.
void emu_error_text(char* out, size_t cap)
{
  std::string s;
  for (const std::string& e : emu::cfg().errors) s += e + "\n";
  if (cap == 0) return;
  const size_t n = s.size() < cap - 1 ? s.size() : cap - 1;
  memcpy(out, s.data(), n);
  out[n] = 0;
}

// the model's own number conversions, exported so that a test can pin them
uint16_t emu_f32_to_f16(float v) { return emu::float_to_f16(v); }
uint16_t emu_f32_to_bf16(float v) { return emu::float_to_bf16(v); }
float emu_f16_to_f32(uint16_t h) { return emu::f16_to_float(h); }

}  // extern "C"
#endif
