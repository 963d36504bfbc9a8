// Pipelined tiled main loop for gfx950 (MI355X): GEMM / batched matmul / implicit-GEMM conv.
//
// One template, one kernel.  The loop structure is the paper's transformed load-and-use loop
// (arXiv 2210.16691, Sec. 4.2 steps 1-5) written by hand for CDNA4:
//   step 1  buffer x S      -> LDS ring of S stages, each [A tile | B tile]; R register slots
//   step 2  index shift     -> iteration ko issues the loads of k-tile ko+S-1
//   step 3  roll and wrap   -> slot = k-tile mod S; k-tiles past the end are issued as
//                              out-of-range buffer loads (they fetch nothing and zero-fill a
//                              free slot), which keeps the number of loads in flight constant
//   step 4  prologue        -> S-1 k-tiles issued before the loop (and, with fusion, the first
//                              fragment read before the loop: Sec. 4.1 step 5)
//   step 5  synchronisation -> producer_commit is implicit (the vector-memory counter counts
//                              loads in issue order); consumer_wait = s_waitcnt vmcnt((S-2)*L)
//                              + s_barrier; consumer_release / producer_acquire = s_waitcnt
//                              lgkmcnt(0) + the same s_barrier of the following iteration.
// Rule 1 of Sec. 3.1 (the buffer must be produced by an asynchronous copy) is met by
// buffer_load_dwordx4 ... lds: data goes HBM/L2 -> LDS without passing through registers.
//
// Data layout in LDS.  A direct-to-LDS load writes lane l's 16 bytes at M0 + 16*l, so the
// LDS image of a tile is linear in (load, wave, lane); the bank-conflict-free swizzle is
// applied on the source side by choosing which 16-byte chunk of the global tile each lane
// fetches (the paper applies shared-memory swizzling to all its kernels, Sec. 6.1).
//   K-contiguous tile (A stored M x K, B stored N x K): rows of BK halves, CPR = BK/8 chunks per
//     row, RPL = 128/BK rows per 256-byte bank line; physical chunk = logical chunk XOR
//     ((row/RPL) mod CPR); read with ds_read_b128.
//   M/N-contiguous tile (A stored K x M, B stored K x N): one row per k, physical chunk =
//     logical chunk XOR (((k/RPB) mod min(4,BX/32)) << 2); read with ds_read_b64_tr_b16,
//     which hands each lane 4 consecutive k of one column (and runs at ~2x the LDS bandwidth
//     of ds_read_b128 on this machine).
//
// Matrix-core mapping.  v_mfma_f32_32x32x16_{f16,bf16} computes D[i][j] += sum_k X[i][k] Y[k][j]
// with X lane l = row l%32, k = 8*(l/32)..+7, Y lane l = column l%32, same k, and D lane l =
// column l%32, rows 8*(v/4) + 4*(l/32) + v%4 for v = 0..15.  We feed X from B (i = n) and Y
// from A (j = m), so a lane owns 4 consecutive n of one output row m: a vector store.
//
// Hardware access.  Every machine-specific operation the loop uses (direct-to-LDS loads, wait
// counters, the barrier, LDS reads, the matrix instruction, global stores) is a static member of
// the policy class HW that the templates below take.  alcop_gfx950.hip.h implements it with
// gfx950 instructions; a test build substitutes a functional model of the same operations and
// runs this very loop on the CPU, one fibre per lane, with bounds checks.  This header contains
// no device intrinsic itself; __global__, __device__, __forceinline__ and __launch_bounds__
// come from the HIP runtime header (or from the test build) that is included before it.

#pragma once
#include <stdint.h>

namespace alcop {

struct Params {
  const void* A;
  const void* B;
  void* C;
  int M, N, K;                 // GEMM view
  int lda, ldb, ldc;           // elements (host guarantees the byte spans fit 31 bits)
  long strideA, strideB, strideC;
  int out_dtype;               // 0 f16, 1 bf16, 2 f32
  int ntm, ntn;                // tile counts
  int raster, group_m;         // block -> tile order
  // convolution geometry (AM != 0): x is NHWC, A rows are (img, p, q)
  int cH, cW, cC, cP, cQ, cS, csh, csw, cph, cpw;
  int cdh, cdw;                // dilation: filter tap (r, s) reads row ih0 + r * cdh, column iw0 + s * cdw
  unsigned a_span, b_span;     // conv: bytes of x; unused otherwise
  // third pipeline level (HBM -> L2): every wave touches lines of k-tile kt + pf_dist when it
  // issues k-tile kt; the lines of a panel are split among the pf_pa (pf_pb) blocks that share it
  int pf_dist, pf_pa, pf_pb;
  // consumer-side fused elementwise function: act(alpha * acc + bias[n])
  float alpha;
  const float* bias;
  int act;
  // split-K kernels (SK == 1): grid.z blocks share an output tile, block z reduces over
  // k in [z * ksplit_len, min(K, (z + 1) * ksplit_len)) and stores its fp32 partial tile at
  // C + z * zstrideC elements (C is then the caller's workspace)
  int ksplit_len;
  long zstrideC;
  // convolution with an LDS-resident input patch (AM == 3): filter height, row length of the
  // zero-padded image, tiles per image, direct-to-LDS loads per thread that bring in the patch
  int cR, cWp, ntj, patch_loads;
  // persistent producer / consumer kernels (alcop_stream.hip.h): blocks launched and batch count;
  // block b works on tiles b, b + sgrid, b + 2 sgrid, ... of the ntm * ntn * sbatch tiles
  int sgrid, sbatch;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Layout of an operand tile, in global memory and (swizzled) in LDS.
enum { LAY_K = 0,    // contiguous along k:            A stored M x K, B stored N x K
       LAY_MN = 1 }; // contiguous along its m or n:   A stored K x M, B stored K x N

// Compile-time description of one operand tile: BX rows/columns of the block tile, WX of them
// per wave, BK deep, moved by NT threads.
template <int LAY_, int BX_, int WX_, int BK_, int NT_>
struct Opnd {
  static constexpr int LAY = LAY_, BX = BX_, WX = WX_, BK = BK_, NT = NT_;
  static constexpr int BYTES = BX * BK * 2;
  // An M/N-contiguous tile whose width is a multiple of 64 but not a power of two (192 = 3 x 64)
  // is kept in LDS as BX / 64 images of 64 columns each, one after the other; each image has
  // the layout and swizzle of a 64-wide tile, and one block-wide load fills exactly one image.
  static constexpr bool PARTS = LAY == LAY_MN && BX % 64 == 0 && (BX & (BX - 1)) != 0;
  static constexpr int PBX = PARTS ? 64 : BX;                  // columns of one LDS image
  static constexpr int ROWB = LAY == LAY_K ? BK * 2 : PBX * 2; // bytes of one LDS row
  static constexpr int CPR = ROWB / 16;                        // 16-byte chunks per LDS row
  static constexpr int RSTEP = NT / CPR;                       // LDS rows one block-wide load covers
  static constexpr int NL = BYTES / (NT * 16);                 // loads per thread and k-tile
  static constexpr int TX = WX / 32;                           // 32-wide sub-tiles per wave
  // swizzle of the M/N-contiguous layout
  static constexpr int UPR = PBX / 32;                         // 64-byte units per row
  static constexpr int RPB = (4 / UPR) > 1 ? (4 / UPR) : 1;    // rows per 256-byte bank line
  static constexpr int GM = UPR < 4 ? UPR : 4;
  static constexpr int NRD = LAY == LAY_K ? BK / 16 : TX;      // lane-address registers of the reader
  static constexpr int NRI = LAY == LAY_K ? TX : 2 * TX;       // LDS read instructions per fragment
  // 128-byte lines (or parts of lines) in the k-slice of one tile, for the L2 touches
  static constexpr int LINES = LAY == LAY_K ? BX : BK * ((BX * 2) / 128);
  static_assert(BYTES % (NT * 16) == 0, "loads per thread");
  static_assert(!PARTS || NT == BK * CPR, "one block-wide load per 64-column image");
  // K-contiguous layout: the LDS has 64 banks of 4 bytes, so RPL = 256 / (row bytes) rows share
  // one 256-byte bank line (4, 2, 1 rows for BK = 32, 64, 128).  A 16-byte read instruction is
  // served 16 lanes (= 16 consecutive rows of one chunk column) per clock; they hit 16 distinct
  // 16-byte bank groups when rows in the same position of consecutive bank lines take different
  // chunks: physical chunk = logical chunk XOR ((row / RPL) mod CPR).
  static constexpr int RPL = (128 / BK) > 1 ? (128 / BK) : 1;
  static_assert(LAY == LAY_K ? (RSTEP % (RPL * CPR) == 0) : (RSTEP % (4 * RPB) == 0), "swizzle period");
  // logical 16-byte chunk -> physical chunk within LDS row `row` (HW::kSwizzle = false, a
  // measurement aid, leaves the tile image unpermuted: same results, bank conflicts)
  template <class HW>
  __device__ static __forceinline__ int swz(int row)
  {
    if constexpr (!HW::kSwizzle) return 0;
    return LAY == LAY_K ? ((row / RPL) % CPR) : (((row / RPB) % GM) << 2);
  }
};

// One kernel = one KCfg.  DT: 0 fp16, 1 bf16 operands.  BM x BN x BK: block tile; WM x WN: wave
// tile.  S: stages of the LDS ring (1 = unpipelined); R: register slots for fragments (2 = the
// inner, LDS -> register pipeline); FUSE: the inner pipeline runs across k-tiles (Fig. 3(d)).
// BL / AL: operand layouts; AM: how the A tile is produced (matrix or convolution gather);
// SK: split-K variant (grid.z slices of the reduction axis, fp32 partial tiles).
// PF: the kernel has the third pipeline level (HBM -> L2 touches, one more load per wave and k-tile).
template <int DT_, int BM_, int BN_, int BK_, int WM_, int WN_, int S_, int R_, int FUSE_,
          int BL_, int AM_, int AL_ = 0, int SK_ = 0, int PF_ = 0>
struct KCfg {
  static constexpr int DT = DT_, BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
  static constexpr int S = S_, R = R_, FUSE = FUSE_, BL = BL_, AM = AM_, AL = AL_, SK = SK_;
  static constexpr int PF = PF_;
  static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN, NWAVES = WAVES_M * WAVES_N;
  static constexpr int NT = NWAVES * 64;
  // AL: 0 = A stored M x K, 1 = A stored K x M.  BL: 0 = B stored K x N, 1 = B stored N x K.
  using OA = Opnd<AL ? LAY_MN : LAY_K, BM, WM, BK, NT>;
  using OB = Opnd<BL ? LAY_K : LAY_MN, BN, WN, BK, NT>;
  static constexpr int TM = WM / 32, TN = WN / 32, NKI = BK / 16;
  // AM == 3 keeps its A operand in a patch outside the ring: a stage holds the B tile only
  static constexpr int A_BYTES = AM == 3 ? 0 : OA::BYTES, B_BYTES = OB::BYTES;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int RING_BYTES = S * STAGE_BYTES;
  static constexpr int EPI_WAVE_BYTES = 32 * (WN * 4 + 16);     // epilogue band, fp32 worst case
  // the kernels with L2 touches add a landing pad per wave; without it two stages of a 40 KB
  // stage are exactly 80 KB and two blocks share a compute unit
  static constexpr int MAIN_BYTES = RING_BYTES + (PF_ ? NWAVES * 256 : 0);
  static constexpr int LDS_BYTES =
      MAIN_BYTES > NWAVES * EPI_WAVE_BYTES ? MAIN_BYTES : NWAVES * EPI_WAVE_BYTES;
  static constexpr int NLA = AM == 3 ? 0 : OA::NL, NLB = OB::NL;
  // AM == 3: the patch follows the ring and the landing pad, 1024-byte aligned; its size depends
  // on the convolution's geometry and is added to the dynamic LDS size at launch
  static constexpr int PATCH_OFF = (MAIN_BYTES + 1023) / 1024 * 1024;
  static constexpr int L = NLA + NLB + PF;  // per wave and k-tile: tile loads (+ one L2 touch)
  static constexpr int WAIT = (S >= 2 ? (S - 2) * L : 0);    // loads allowed in flight at a wait
  static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "wave tile");
  static_assert(BK == 32 || BK == 64 || BK == 128, "bk");
  static_assert(S >= 1 && S <= 4 && R >= 1 && R <= 4, "stages");
  static_assert(!FUSE || (R >= 2 && S >= 2), "fusion needs a register double buffer and S>=2");
  // R >= 3: R - 1 fragments are in flight ahead of the one the matrix cores consume.  They may
  // reach into the next k-tile but not beyond it, and only the fused pipeline is built that deep.
  static_assert(R <= 2 || (FUSE && R - 1 <= BK / 16), "deep register pipeline");
  // loads allowed in flight when the prologue of the deep pipeline, which primes all S slots,
  // waits for k-tile 0 (a smaller number than necessary only waits for more)
  static constexpr int WAIT0 = (S - 1) * L < 63 ? (S - 1) * L : 63;
  // AM: 0 = A is a matrix; 1 = A is gathered from an NHWC image and a k-tile lies inside one
  // filter tap (bk divides the channel count: the tap is the same for all lanes); 2 = gathered,
  // any channel count that is a multiple of 8 (every lane tracks the tap of its own chunk);
  // 3 = stride-1 convolution with C = BK whose input patch (tile + halo) is loaded into LDS once
  // and whose filter taps are formed by shifted LDS reads: only the weights stream through the ring
  static_assert(AM != 3 || (SK == 0 && BL == 0), "patch convolution: RSCK weights, no split-K");
  static_assert(!PF || (AM == 0 && SK == 0 && FUSE), "L2 touches: fused matrix-operand kernels only");
  static_assert(!PF || !(OA::PARTS || OB::PARTS), "L2 touches: tile widths that are powers of two");
  static_assert(!(AM != 0 && AL == 1), "the convolution gather produces a K-contiguous A tile");
  static_assert(WAIT <= 63, "vmcnt is a 6-bit counter");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS ring exceeds 160 KB");
};

// Dynamic LDS bytes a launch of configuration C needs (host side).
template <class C>
inline int dynamic_lds_bytes(const Params& p)
{
  if constexpr (C::AM == 3) {
    const int need = C::PATCH_OFF + p.patch_loads * C::NT * 16;
    return need > C::LDS_BYTES ? need : C::LDS_BYTES;
  } else {
    return C::LDS_BYTES;
  }
}

// Per-lane state of the producer side of one operand.
template <class HW>
struct LoadState {
  typename HW::Rsrc rsrc;
  uint32_t voff;     // byte offset of this lane's chunk in load 0 of k-tile 0
  uint32_t voff_t;   // the same for a partial last k-tile (out of range if the chunk is past K)
  uint32_t step;     // byte distance between consecutive loads of one k-tile
  uint32_t kstep;    // byte distance between consecutive k-tiles
};

// Producer set-up.  `ptr` is the operand of this batch entry, `t` the tile index along the
// operand's own dimension, `extent` its size there (M or N), `ld` the leading dimension.
// Lane q0 of the block owns 16-byte LDS slot q0 (+ NT per further load); which global chunk it
// fetches follows from the swizzle.  The descriptor covers exactly the valid part of the
// operand seen from the tile's origin, so rows / columns / k beyond it read as zero.
template <class O, class HW>
__device__ __forceinline__ LoadState<HW> setup_loader(const void* ptr, int t, int extent, int ld,
                                                      int K, int nko, int q0)
{
  LoadState<HW> st;
  const int r = q0 / O::CPR, ph = q0 % O::CPR;
  const int c = ph ^ O::template swz<HW>(r);
  const int valid = (extent - t * O::BX) < O::BX ? (extent - t * O::BX) : O::BX;
  if constexpr (O::LAY == LAY_K) {
    const char* base = (const char*)ptr + (long)t * O::BX * ld * 2;
    st.rsrc = HW::make_rsrc(base, ((valid - 1) * ld + K) * 2);
    st.voff = (uint32_t)(r * ld * 2 + c * 16);
    st.step = (uint32_t)(O::RSTEP * ld * 2);
    st.kstep = O::BK * 2;
    st.voff_t = ((nko - 1) * O::BK + c * 8 >= K) ? (st.voff | 0x80000000u) : st.voff;
  } else {
    const char* base = (const char*)ptr + (long)t * O::BX * 2;
    st.rsrc = HW::make_rsrc(base, ((K - 1) * ld + valid) * 2);
    st.voff = (uint32_t)(r * ld * 2 + c * 16);
    // the next load: RSTEP rows further down, or (64-column images) the same rows of the next image
    st.step = O::PARTS ? (uint32_t)(O::PBX * 2) : (uint32_t)(O::RSTEP * ld * 2);
    st.kstep = (uint32_t)(O::BK * ld * 2);
    st.voff_t = st.voff;   // rows k >= K lie beyond the descriptor
  }
  return st;
}

// Consumer set-up: lane addresses (relative to the stage base) of the operand fragment that
// feeds v_mfma_f32_32x32x16: lane l = row/column l%32 of a 32-wide sub-tile, k = 8*(l/32)..+7.
template <class O, class HW>
__device__ __forceinline__ void setup_reader(int lane, int wx, uint32_t tile_off,
                                             uint32_t (&rd)[O::NRD])
{
  if constexpr (O::LAY == LAY_K) {
    const int row = wx * O::WX + (lane & 31);
#pragma unroll
    for (int ki = 0; ki < O::NRD; ki++)
      rd[ki] = tile_off + (uint32_t)(row * (O::BK * 2) + (((2 * ki + (lane >> 5)) ^ O::template swz<HW>(row)) * 16));
  } else {
    // transposing read: 16-lane group G reads 4 k-rows x 16 columns; lane s of the group
    // supplies row s/4, columns 4*(s%4)..+3 and receives column s, rows 0..3.
    const int G = lane >> 4, s = lane & 15;
    const int k = 8 * (G >> 1) + (s >> 2);
#pragma unroll
    for (int t = 0; t < O::NRD; t++) {
      const int n = wx * O::WX + t * 32 + 16 * (G & 1) + 4 * (s & 3);
      const int img = n / O::PBX, nl = n % O::PBX;          // image 0 and n itself unless PARTS
      const int c = (nl >> 3) ^ O::template swz<HW>(k);
      rd[t] = tile_off + (uint32_t)(img * (O::BK * O::ROWB) + k * O::ROWB + c * 16 + (n & 7) * 2);
    }
  }
}

// LDS read instruction r (0 <= r < O::NRI) of fragment ki; cur[] = slot base + lane addresses.
template <class O, class HW>
__device__ __forceinline__ void read_instr(const uint32_t (&cur)[O::NRD], int ki, int r,
                                           u32x4 (&frag)[O::TX])
{
  if constexpr (O::LAY == LAY_K) {
    frag[r] = HW::lds_read16(cur[ki] + r * (32 * O::BK * 2));
  } else {
    const int t = r >> 1, h = r & 1;
    const u32x2 v = HW::lds_read_tr8(cur[t] + ki * (16 * O::ROWB) + h * (4 * O::ROWB));
    frag[t][2 * h] = v[0];
    frag[t][2 * h + 1] = v[1];
  }
}

// Address of the 128-byte line that lane j of an operand's L2-touch share owns in k-tile 0, and
// the byte step from one k-tile to the next.  The lines of the tile's k-slice are dealt round
// robin to the `sharers` blocks that load the same panel; `me` is this block's index among them.
// Returns false when lane j has no line.
template <class O>
__device__ __forceinline__ bool touch_line(const void* ptr, int t, int extent, int ld, int j,
                                           int sharers, int me, const char** out, uint32_t* kstep)
{
  if constexpr (O::LAY == LAY_K) {
    if (j >= O::LINES / sharers) return false;
    int row = j * sharers + me;
    if (t * O::BX + row >= extent) row = 0;
    *out = (const char*)ptr + ((long)t * O::BX + row) * ld * 2;
    *kstep = O::BK * 2;
  } else {
    constexpr int LPR = (O::BX * 2) / 128;                  // lines per k-row of the tile
    if (j >= O::LINES / sharers) return false;
    const int line = j * sharers + me;
    const int row = line / LPR;
    int seg = line % LPR;
    if (t * O::BX + seg * 64 >= extent) seg = 0;
    *out = (const char*)ptr + ((long)row * ld + (long)t * O::BX + seg * 64) * 2;
    *kstep = (uint32_t)(O::BK * ld * 2);
  }
  return true;
}

template <class C, class HW>
__global__ void __launch_bounds__(C::NT) alcop_mainloop(const Params p)
{
  constexpr int BM = C::BM, BN = C::BN, BK = C::BK, WM = C::WM, WN = C::WN, S = C::S;
  constexpr int TM = C::TM, TN = C::TN, NKI = C::NKI, NLA = C::NLA, NLB = C::NLB;
  constexpr int NWAVES = C::NWAVES, STAGE_BYTES = C::STAGE_BYTES, A_BYTES = C::A_BYTES;

  const uint32_t lds0 = HW::lds_base();      // dynamic LDS of the block, 1024-byte aligned

  const int lane = HW::lane_id();
  const int wave = HW::wave_id();
  const int wm = wave % C::WAVES_M, wn = wave / C::WAVES_M;
  const int batch = HW::block_y();

  // ---- block -> tile (paper Sec. 1: inter-tile parallelism; the order only affects L2 reuse)
  int lid = HW::block_x();
  const int nblk = p.ntm * p.ntn;
  int tm, tn;
  if (p.raster == 1) {
    if ((nblk & 7) == 0) lid = (lid & 7) * (nblk >> 3) + (lid >> 3);   // blocks of one XCD adjacent
    const int width = p.group_m * p.ntn;
    const int g = lid / width;
    const int first = g * p.group_m;
    const int gsz = (p.ntm - first) < p.group_m ? (p.ntm - first) : p.group_m;
    const int rem = lid - g * width;
    tm = first + rem % gsz;
    tn = rem / gsz;
  } else {
    tm = lid / p.ntn;
    tn = lid - tm * p.ntn;
  }
  // the k range of this block: all of K, or one slice of it (split-K; slices are whole k-tiles)
  int k0 = 0, Kb = p.K;
  if constexpr (C::SK) {
    k0 = (int)HW::block_z() * p.ksplit_len;
    Kb = (p.K - k0) < p.ksplit_len ? (p.K - k0) : p.ksplit_len;
  }
  const int nko = (Kb + BK - 1) / BK;         // the last k-tile may be partial (K % 8 == 0)
  const bool ktail = (Kb % BK) != 0;

  // ---- global -> LDS producers -----------------------------------------------------------
  using OA = typename C::OA;
  using OB = typename C::OB;
  const int q0 = wave * 64 + lane;            // 16-byte LDS slot of this lane in load 0
  const char* Abatch = (const char*)p.A + (long)batch * p.strideA * 2;
  const char* Bbatch = (const char*)p.B + (long)batch * p.strideB * 2;
  if constexpr (C::SK) {   // origin of the slice: k0 columns (k-contiguous) or k0 rows further
    if constexpr (C::AM == 0) Abatch += (long)k0 * (C::AL ? p.lda : 1) * 2;
    Bbatch += (long)k0 * (C::BL ? 1 : p.ldb) * 2;
  }
  LoadState<HW> la, lb;
  // convolution: per-load row geometry of the gathered A tile
  int ih0[NLA > 0 ? NLA : 1], iw0[NLA > 0 ? NLA : 1];
  uint32_t coff[NLA > 0 ? NLA : 1];
  int cr = 0, cs = 0, cc0 = 0;                // (r, s, c0) of the next k-tile to issue
  int crd = 0, csd = 0;                       // r * dilation_h, s * dilation_w of that tap
  bool a_in_k = true;                         // AM == 2: this lane's chunk lies below K
  int a_k8 = 0;                               // AM == 2: k of this lane's chunk within a k-tile
  if constexpr (C::SK && C::AM == 1) {        // the slice starts at tap k0 / C, channel k0 % C
    const int tap = k0 / p.cC;
    cc0 = k0 - tap * p.cC;
    cr = tap / p.cS;
    cs = tap - cr * p.cS;
    crd = cr * p.cdh;
    csd = cs * p.cdw;
  }
  // AM == 3: the tile is BM consecutive positions j of one image's output space laid out with
  // the padded row length Wp (positions with column >= Q are computed and not stored); for
  // filter tap (r, s) the A operand is the same patch shifted by r * Wp + s rows
  int p_img = 0, p_j0 = 0;
  const uint32_t patch_base = lds0 + C::PATCH_OFF;
  if constexpr (C::AM == 0) {
    la = setup_loader<OA, HW>(Abatch, tm, p.M, p.lda, Kb, nko, q0);
  } else if constexpr (C::AM == 3) {
    p_img = tm / p.ntj;
    p_j0 = (tm - p_img * p.ntj) * BM;
    la.rsrc = HW::make_rsrc(p.A, (int)p.a_span);
    la.voff = la.voff_t = la.step = la.kstep = 0;
    const int rows = BM + (p.cR - 1) * p.cWp + (p.cS - 1);       // patch rows = tile + halo
    for (int i = 0; i < p.patch_loads; i++) {
      // 16-byte slot q of the patch: row q / CPR, physical chunk q % CPR (swizzled like any
      // k-contiguous tile); rows are positions of the padded image, zero outside the image
      const int q = q0 + i * C::NT;
      const int row = q / OA::CPR;
      const int c = (q % OA::CPR) ^ OA::template swz<HW>(row);
      const int jj = p_j0 + row;
      const int ihp = jj / p.cWp;
      const int ih = ihp - p.cph, iw = jj - ihp * p.cWp - p.cpw;
      const bool ok = row < rows && (unsigned)ih < (unsigned)p.cH && (unsigned)iw < (unsigned)p.cW;
      const uint32_t off = (uint32_t)((((p_img * p.cH + ih) * p.cW) + iw) * p.cC * 2 + c * 16);
      HW::dma16(la.rsrc, ok ? off : 0x80000000u, patch_base + (uint32_t)(i * C::NT + wave * 64) * 16u);
    }
  } else {
    // implicit GEMM: row m of A is output pixel (img, p, q); a k-tile lies inside one filter tap
    // (r, s) because bk divides C, so a lane's chunk is 16 contiguous bytes of x or padding.
    la.rsrc = HW::make_rsrc(p.A, (int)p.a_span);
    la.voff = la.voff_t = la.step = la.kstep = 0;
    const int r = q0 / OA::CPR, ph = q0 % OA::CPR;
    const int c = ph ^ OA::template swz<HW>(r);
    if constexpr (C::AM == 2) {
      // C is any multiple of 8: a chunk of 8 channels still lies inside one tap, but the chunks
      // of a k-tile may belong to different taps, so (r, s, c0) are per lane and start at the
      // lane's own k
      a_k8 = c * 8;
      const int kc = k0 + a_k8;
      const int tap = kc / p.cC;
      cc0 = kc - tap * p.cC;
      cr = tap / p.cS;
      cs = tap - cr * p.cS;
      crd = cr * p.cdh;
      csd = cs * p.cdw;
    }
#pragma unroll
    for (int i = 0; i < NLA; i++) {
      const int m = tm * BM + r + i * OA::RSTEP;
      const int img = m / (p.cP * p.cQ);
      const int pq = m - img * (p.cP * p.cQ);
      const int pp = pq / p.cQ, qq = pq - pp * p.cQ;
      ih0[i] = (m < p.M) ? pp * p.csh - p.cph : -0x40000000;
      iw0[i] = qq * p.csw - p.cpw;
      coff[i] = (uint32_t)((((img * p.cH + (pp * p.csh - p.cph)) * p.cW) + iw0[i]) * p.cC * 2 +
                           (C::AM == 2 ? 0 : c * 16));
    }
  }
  lb = setup_loader<OB, HW>(Bbatch, tn, p.N, p.ldb, Kb, nko, q0);

  // ---- HBM -> L2 touches (third pipeline level) --------------------------------------------
  // The blocks of one XCD that run side by side load the same A row-panel (those with equal tm)
  // or B column-panel (equal tn) at about the same time, so each line misses L2 once and all
  // sharers wait for that miss.  Touching the line pf_dist k-tiles earlier, once, by one of the
  // sharers, turns the tile loads into L2 hits.  Lane x of the block owns one line per k-tile.
  int pf_d = 0;
  const char* pf_ptr = Bbatch;                // a valid address for lanes without a line
  uint32_t pf_step = 0;
  if constexpr (C::PF) {
    pf_d = p.pf_dist < nko - 1 ? p.pf_dist : nko - 1;   // never past the last k-tile
    if (pf_d > 0) {
      const int na = (C::AM == 0) ? OA::LINES / p.pf_pa : 0;   // lines of A this block touches
      bool have = false;
      if constexpr (C::AM == 0)
        have = touch_line<OA>(Abatch, tm, p.M, p.lda, q0, p.pf_pa, tn % p.pf_pa, &pf_ptr, &pf_step);
      if (!have && q0 >= na)
        have = touch_line<OB>(Bbatch, tn, p.N, p.ldb, q0 - na, p.pf_pb, tm % p.pf_pb, &pf_ptr, &pf_step);
      if (!have) {
        pf_ptr = Bbatch;
        pf_step = 0;
      }
      pf_ptr += (long)pf_step * pf_d;
    }
  }
  const uint32_t pf_dst = lds0 + C::RING_BYTES + (uint32_t)wave * 256u;

  // Loads of one k-tile: stage_begin fixes the wave-uniform offsets of k-tile `kt` and ring slot
  // `slot`; issue_one(i) emits load i of the L loads a wave owns (A loads, B loads, and the L2
  // touch of the kernels that have that level);
  // stage_end advances the convolution tap.  Always exactly L loads per wave and stage.
  // A partial last k-tile selects the lane offsets that zero-fill chunks at k >= K: one select
  // per operand and k-tile, nothing per load.
  uint32_t st_ka = 0, st_kb = 0, st_dst = 0, st_tap = 0;
  uint32_t st_voffA = la.voff, st_voffB = lb.voff;
  bool st_live = false, st_pf_live = false;
  auto stage_begin = [&](int kt, int slot) {
    st_live = kt < nko;
    const bool tail = ktail && kt == nko - 1;
    st_voffA = tail ? la.voff_t : la.voff;
    st_voffB = tail ? lb.voff_t : lb.voff;
    st_pf_live = kt + pf_d + 1 < nko;
    st_dst = lds0 + (uint32_t)slot * STAGE_BYTES + (uint32_t)wave * 1024u;
    if constexpr (C::AM == 0)
      st_ka = st_live ? (uint32_t)kt * la.kstep : 0x80000000u;
    else if constexpr (C::AM != 3)
      st_tap = (uint32_t)(((crd * p.cW + csd) * p.cC + cc0) * 2);
    if constexpr (C::AM == 2) a_in_k = kt * BK + a_k8 < Kb;
    st_kb = st_live ? (uint32_t)kt * lb.kstep : 0x80000000u;
  };
  auto issue_one = [&](int idx) {
    if (idx < NLA) {
      const int i = idx;
      if constexpr (C::AM == 0) {
        HW::dma16(la.rsrc, st_voffA + st_ka + (uint32_t)i * la.step, st_dst + i * (NWAVES * 1024));
      } else {
        bool ok = st_live && (unsigned)(ih0[i] + crd) < (unsigned)p.cH &&
                  (unsigned)(iw0[i] + csd) < (unsigned)p.cW;
        if constexpr (C::AM == 2) ok = ok && a_in_k;
        HW::dma16(la.rsrc, ok ? coff[i] + st_tap : 0x80000000u, st_dst + i * (NWAVES * 1024));
      }
    } else if (idx < NLA + NLB) {
      const int i = idx - NLA;
      HW::dma16(lb.rsrc, st_voffB + st_kb + (uint32_t)i * lb.step,
            st_dst + A_BYTES + i * (NWAVES * 1024));
    } else if constexpr (C::PF) {
      HW::touch4(pf_ptr, pf_dst);
      if (st_pf_live) pf_ptr += pf_step;      // stop at the last k-tile: never run past the operand
    }
  };
  auto stage_end = [&]() {
    if constexpr (C::AM == 1) {
      cc0 += BK;
      if (cc0 == p.cC) {
        cc0 = 0; cs++; csd += p.cdw;
        if (cs == p.cS) { cs = 0; csd = 0; cr++; crd += p.cdh; }
      }
    }
    if constexpr (C::AM == 2) {
      cc0 += BK;
      while (cc0 >= p.cC) {
        cc0 -= p.cC; cs++; csd += p.cdw;
        if (cs == p.cS) { cs = 0; csd = 0; cr++; crd += p.cdh; }
      }
    }
  };
  auto issue = [&](int kt, int slot) {
    stage_begin(kt, slot);
#pragma unroll
    for (int i = 0; i < C::L; i++) issue_one(i);
    stage_end();
  };

  // ---- LDS -> register consumers ---------------------------------------------------------
  // Y operand (matrix-core column operand) from A, X operand (row operand) from B.  Lane
  // addresses are fixed per kernel; cur* = slot base + lane address is refreshed once per
  // k-tile so that every read is "register + immediate".
  uint32_t rdA[OA::NRD], rdB[OB::NRD];
  setup_reader<OA, HW>(lane, wm, 0, rdA);
  setup_reader<OB, HW>(lane, wn, A_BYTES, rdB);
  uint32_t curA[OA::NRD], curB[OB::NRD];
  int tap_r = 0, tap_s = 0, tap_n = 0;        // AM == 3: filter tap of the k-tile read next
  auto set_read_slot = [&](uint32_t sbase) {
    if constexpr (C::AM == 3) {
      // one k-tile per tap (C = BK): the fragment rows are the wave's rows shifted by the tap;
      // the read past the last k-tile (fused pipeline) is pointed at the unshifted rows
      const int shift = tap_n < nko ? tap_r * p.cWp + tap_s : 0;
      const int row = wm * WM + (lane & 31) + shift;
#pragma unroll
      for (int ki = 0; ki < OA::NRD; ki++)
        curA[ki] = patch_base + (uint32_t)(row * (BK * 2) + (((2 * ki + (lane >> 5)) ^ OA::template swz<HW>(row)) * 16));
      tap_n++;
      if (++tap_s == p.cS) { tap_s = 0; tap_r++; }
    } else {
#pragma unroll
      for (int i = 0; i < OA::NRD; i++) curA[i] = sbase + rdA[i];
    }
#pragma unroll
    for (int i = 0; i < OB::NRD; i++) curB[i] = sbase + rdB[i];
  };
  // LDS read instruction r of fragment ki: the A reads come first, then the B reads.
  constexpr int NRI = OA::NRI + OB::NRI;
  auto read_one = [&](int ki, int r, u32x4(&fa)[TM], u32x4(&fb)[TN]) {
    if (r < OA::NRI)
      read_instr<OA, HW>(curA, ki, r, fa);
    else
      read_instr<OB, HW>(curB, ki, r - OA::NRI, fb);
  };
  auto load_frags = [&](int ki, u32x4(&fa)[TM], u32x4(&fb)[TN]) {
#pragma unroll
    for (int r = 0; r < NRI; r++) read_one(ki, r, fa, fb);
  };

  f32x16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; i++)
#pragma unroll
    for (int j = 0; j < TM; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  // One register-level step: the TN*TM matrix instructions on fragment (ua, ub); the LDS reads
  // of the next fragment (if nread) are issued two per matrix instruction starting right after
  // instruction `first`, so that they have returned long before the step ends; the
  // direct-to-LDS loads [d0, d1) of the k-tile being fetched are spread evenly.  `first` > 0
  // leaves room for the block-wide synchronisation that `sync` performs after instruction
  // first-1.  The compiler must keep exactly this order (sched_barrier).
  constexpr int NMM = TM * TN;
  auto step = [&](u32x4(&ua)[TM], u32x4(&ub)[TN], bool nread, int nki, u32x4(&na)[TM],
                  u32x4(&nb)[TN], int d0, int d1, int first, auto&& sync) {
    const int gaps = NMM - first > 0 ? NMM - first : 1;
    const int rpg = (NRI + gaps - 1) / gaps > 2 ? (NRI + gaps - 1) / gaps : 2;   // reads per gap
#pragma unroll
    for (int m = 0; m < NMM; m++) {
      const int i = m / TM, j = m % TM;
      acc[i][j] = HW::template mma<C::DT>(ub[i], ua[j], acc[i][j]);
      if (m + 1 == first || (first >= NMM && m == NMM - 1)) sync();
      if (nread && (m >= first || m == NMM - 1)) {
        const int g = m >= first ? m - first : 0;
#pragma unroll
        for (int r = g * rpg; r < (g + 1) * rpg && r < NRI; r++) read_one(nki, r, na, nb);
      }
#pragma unroll
      for (int d = d0 + m * (d1 - d0) / NMM; d < d0 + (m + 1) * (d1 - d0) / NMM; d++) issue_one(d);
      HW::sched_fence();
    }
  };
  auto no_sync = [] {};

  u32x4 fa[C::R][TM], fb[C::R][TN];

  // ---- the pipelined main loop -----------------------------------------------------------
  if constexpr (C::FUSE && C::R >= 3) {
    // Deep holistic pipeline (Table 1: the stage count of the register-level pipeline is a free
    // parameter; Fig. 3(d) fusion).  D = R-1 fragments are being read ahead of the fragment the
    // matrix cores consume, so that an LDS read has at least D-1 whole steps to return; with one
    // wave per SIMD nothing else hides that latency.  The loop runs in periods: period p opens
    // with the block-wide synchronisation after which k-tile p+1 may be read and the slot of
    // k-tile p may be refilled; its step t reads fragment t of k-tile p+1 and computes fragment
    // KS+t of k-tile p (continuing into k-tile p+1 when KS+t >= NKI).  The ring is primed with
    // S k-tiles; k-tile p+S is issued during steps 1..NKI-1 of period p.
    constexpr int R = C::R, D = R - 1, KS = NKI - D;
    constexpr int G = (NKI % R == 0) ? R : ((NKI % 2 == 0 && R % 2 == 0) ? 2 : 1);   // gcd(NKI, R)
    constexpr int U = R / G;                  // periods per unrolled body: register slots are static
#pragma unroll
    for (int s = 0; s < S; s++) issue(s, s);
    HW::template wait_vm<C::WAIT0>();
    HW::block_barrier();
    set_read_slot(lds0);
#pragma unroll
    for (int d = 0; d < D; d++) load_frags(d, fa[d], fb[d]);
    HW::sched_fence();
    // steps 0..KS-1 of k-tile 0: the rest of its fragments are read, nothing is issued
#pragma unroll
    for (int ki = 0; ki < KS; ki++)
      step(fa[ki % R], fb[ki % R], true, ki + D, fa[(ki + D) % R], fb[(ki + D) % R], 0, 0, 0, no_sync);
    int rslot = 0, wslot = 0;
    bool done = false;
    for (int p0 = 0; p0 < nko && !done; p0 += U) {
#pragma unroll
      for (int u = 0; u < U; u++) {
        const int pp = p0 + u;
        if (U > 1 && pp >= nko) break;
        const bool last = pp + 1 == nko;
#pragma unroll
        for (int t = 0; t < NKI; t++) {
          // fragment u*NKI + KS + t (counted from the body's first period) is consumed, the one D
          // later is read; past the last k-tile only the consuming steps t < D remain
          const int cs = (u * NKI + KS + t) % R, rs = (u * NKI + KS + t + D) % R;
          if (t >= D && last) { done = true; break; }
          if (t == 0) {
            constexpr int FIRST = NMM >= 8 ? NMM / 4 : 1;
            step(fa[cs], fb[cs], true, 0, fa[rs], fb[rs], 0, 0, FIRST, [&] {
              HW::template wait_vm<C::WAIT>();   // consumer_wait: k-tile p+1 has landed (this wave)
              HW::wait_lds();                    // consumer_release: my reads of k-tile p are done
              HW::block_barrier();               // ... for every wave
              stage_begin(pp + S, wslot);        // the slot of k-tile p is refilled with k-tile p+S
              wslot = (wslot + 1 == S) ? 0 : wslot + 1;
              rslot = (rslot + 1 == S) ? 0 : rslot + 1;
              set_read_slot(lds0 + rslot * STAGE_BYTES);
            });
          } else {
            step(fa[cs], fb[cs], true, t, fa[rs], fb[rs], (t - 1) * C::L / (NKI - 1),
                 t * C::L / (NKI - 1), 0, no_sync);
          }
        }
        if (done) break;
        stage_end();
      }
    }
  } else if constexpr (C::FUSE) {
    // Holistic pipeline over (ko, ki): Fig. 3(d).  The loads of k-tile ko+S-1 are issued during
    // steps 0..NKI-2; the wait for k-tile ko+1 and the barrier open step NKI-1, whose reads
    // already fetch the first fragment of k-tile ko+1.
#pragma unroll
    for (int s = 0; s < S - 1; s++) issue(s, s);
    HW::template wait_vm<C::WAIT>();
    HW::block_barrier();
    set_read_slot(lds0);
    load_frags(0, fa[0], fb[0]);
    int rslot = 0, wslot = S - 1;
    for (int ko = 0; ko < nko; ko++) {
      stage_begin(ko + S - 1, wslot);
      wslot = (wslot + 1 == S) ? 0 : wslot + 1;
#pragma unroll
      for (int ki = 0; ki < NKI; ki++) {
        if (ki == NKI - 1) {
          // the synchronisation sits after the first quarter of this step's matrix instructions
          constexpr int FIRST = NMM >= 8 ? NMM / 4 : 1;
          step(fa[ki & 1], fb[ki & 1], true, 0, fa[(ki + 1) & 1], fb[(ki + 1) & 1], 0, 0, FIRST, [&] {
            HW::template wait_vm<C::WAIT>();          // consumer_wait: k-tile ko+1 has landed (this wave)
            HW::wait_lds();                  // consumer_release: my reads of slot ko are done
            HW::block_barrier();             // ... for every wave
            rslot = (rslot + 1 == S) ? 0 : rslot + 1;
            set_read_slot(lds0 + rslot * STAGE_BYTES);
          });
        } else {
          step(fa[ki & 1], fb[ki & 1], true, ki + 1, fa[(ki + 1) & 1], fb[(ki + 1) & 1],
               ki * C::L / (NKI - 1), (ki + 1) * C::L / (NKI - 1), 0, no_sync);
        }
      }
      stage_end();
    }
  } else {
    if constexpr (S >= 2) {
#pragma unroll
      for (int s = 0; s < S - 1; s++) issue(s, s);
    }
    int rslot = 0, wslot = (S >= 2) ? S - 1 : 0;
    for (int ko = 0; ko < nko; ko++) {
      if constexpr (S >= 2) {
        HW::template wait_vm<C::WAIT>();              // consumer_wait for k-tile ko
        HW::wait_lds();
        HW::block_barrier();                 // also releases slot (ko-1) mod S
        stage_begin(ko + S - 1, wslot);  // its loads are spread over the steps below
      } else {
        HW::wait_lds();
        HW::block_barrier();                 // producer_acquire: slot 0 is free
        issue(ko, 0);
        HW::template wait_vm<0>();                    // consumer_wait
        HW::block_barrier();
      }
      wslot = (wslot + 1 == S) ? 0 : wslot + 1;
      set_read_slot(lds0 + rslot * STAGE_BYTES);
      rslot = (rslot + 1 == S) ? 0 : rslot + 1;
      constexpr int DL = (S >= 2) ? C::L : 0;   // loads to interleave (none when S = 1)
      if constexpr (C::R == 2) {
        // register-level pipeline restarted in every ko: Fig. 3(c)
        load_frags(0, fa[0], fb[0]);
        HW::sched_fence();
#pragma unroll
        for (int ki = 0; ki < NKI; ki++)
          step(fa[ki & 1], fb[ki & 1], ki + 1 < NKI, (ki + 1) % NKI, fa[(ki + 1) & 1],
               fb[(ki + 1) & 1], ki * DL / NKI, (ki + 1) * DL / NKI, 0, no_sync);
      } else {
        // single-level: load a fragment, then use it (Fig. 3(b))
#pragma unroll
        for (int ki = 0; ki < NKI; ki++) {
          load_frags(ki, fa[0], fb[0]);
          HW::sched_fence();
          step(fa[0], fb[0], false, 0, fa[0], fb[0], ki * DL / NKI, (ki + 1) * DL / NKI, 0, no_sync);
        }
      }
      if constexpr (S >= 2) stage_end();
    }
  }
  HW::template wait_vm<0>();   // drain the zero-fill loads of the ring's tail before the ring is reused
  HW::wait_lds();
  HW::block_barrier();   // every wave has finished reading the ring

  // ---- epilogue: convert, transpose through LDS, store rows (Table 1, epilogue term) --------
  // A lane holds 4 consecutive n of one row m (16 such groups per 32x32 sub-tile); stored as is,
  // a wave instruction would scatter 8-byte pieces over 32 rows.  Each wave instead parks one
  // 32-row band of its tile in its own LDS region (row stride padded by 16 B) and reads it back
  // with 16 bytes per lane along the row, so every global store covers whole 128-byte lines.
  auto epilogue = [&](auto zero) {
    using OT = decltype(zero);
    constexpr int OB = sizeof(OT);
    constexpr int RS = WN * OB + 16;                 // LDS row stride of the band
    constexpr int LPR = WN * OB / 16;                // lanes per row when reading back
    constexpr int RPI = 64 / LPR;                    // rows per read instruction
    typedef OT ot4 __attribute__((ext_vector_type(4)));
    const uint32_t ebase = lds0 + (uint32_t)wave * C::EPI_WAVE_BYTES;
    const int m0 = tm * BM + wm * WM, n0 = tn * BN + wn * WN;
    char* Cb = (char*)p.C + (long)batch * p.strideC * OB;
    if constexpr (C::SK) Cb += (long)HW::block_z() * p.zstrideC * OB;
    const bool fused = p.alpha != 1.0f || p.bias != nullptr || p.act != 0;
#pragma unroll
    for (int j = 0; j < TM; j++) {
#pragma unroll
      for (int i = 0; i < TN; i++)
#pragma unroll
        for (int vq = 0; vq < 4; vq++) {
          f32x4 v = {acc[i][j][4 * vq + 0], acc[i][j][4 * vq + 1], acc[i][j][4 * vq + 2],
                     acc[i][j][4 * vq + 3]};
          if (fused) {   // f(.) on the accumulators (paper Sec. 3.2: fused into the consumer)
            const int n = n0 + i * 32 + 8 * vq + 4 * (lane >> 5);
            f32x4 b = {0.f, 0.f, 0.f, 0.f};
            if (p.bias != nullptr && n < p.N) b = HW::global_load_f32x4(p.bias + n);
#pragma unroll
            for (int e = 0; e < 4; e++) {
              float t = v[e] * p.alpha + b[e];
              v[e] = (p.act == 1 && t < 0.f) ? 0.f : t;
            }
          }
          const ot4 h = {HW::template cvt<OT>(v[0]), HW::template cvt<OT>(v[1]),
                         HW::template cvt<OT>(v[2]), HW::template cvt<OT>(v[3])};
          HW::lds_write(ebase + (lane & 31) * RS + (i * 32 + 8 * vq + 4 * (lane >> 5)) * OB, h);
        }
      // a row is LPR lanes long; when that does not divide 64 (a wave tile 96 wide) the last
      // lanes of an instruction idle and the last instruction covers fewer rows
      constexpr bool EVEN = 64 % LPR == 0 && 32 % RPI == 0;
      constexpr int NIT = (32 + RPI - 1) / RPI;
#pragma unroll
      for (int t = 0; t < NIT; t++) {
        int r = t * RPI + lane / LPR;
        const int c16 = lane % LPR;
        bool lane_ok = true;
        if constexpr (!EVEN) {
          lane_ok = lane < RPI * LPR && r < 32;
          if (!lane_ok) r = 0;            // every lane takes part in the read; idle ones store nothing
        }
        const u32x4 v = HW::lds_read16(ebase + r * RS + c16 * 16);
        int m = m0 + j * 32 + r;
        const int n = n0 + c16 * (16 / OB);
        bool row_ok = m < p.M;
        if constexpr (C::AM == 3) {
          // position of the padded output space -> output pixel; columns >= Q are not stored
          const int jj = p_j0 + wm * WM + j * 32 + r;
          const int pp = jj / p.cWp, qq = jj - pp * p.cWp;
          row_ok = pp < p.cP && qq < p.cQ;
          m = (p_img * p.cP + pp) * p.cQ + qq;
        }
        if (lane_ok && row_ok && n < p.N)
          HW::global_store16(Cb + ((long)m * p.ldc + n) * OB, v);
      }
    }
  };
  if (p.out_dtype == 2)
    epilogue(0.0f);
  else if (p.out_dtype == 0)
    epilogue((_Float16)0);
  else
    epilogue((__bf16)0);
}

}  // namespace alcop
