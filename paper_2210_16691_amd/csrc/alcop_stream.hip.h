// Persistent, producer / consumer form of the pipelined loop: the load-and-use pipeline of the
// paper (arXiv 2210.16691, Sec. 1 and Fig. 2: loads of later chunks overlap the use of earlier
// ones) carried ACROSS output tiles.
//
// Why.  The tile-at-a-time kernel starts every block with an empty pipeline and ends it with an
// epilogue during which nothing is in flight.  For outputs with a short reduction axis (the
// paper notes that those "cannot amortize" the initial loads, Sec. 6.1: attention's Q.K^T has one
// or two k-tiles per tile) and for tile counts that do not fill the machine evenly, that fill and
// drain time is most of the run.  Here a block stays on its compute unit and walks a list of
// tiles (tile = block index + j * blocks launched); its k-tiles form ONE stream through the
// S-stage LDS ring, so the loads of the next tile are in flight while the current tile is
// multiplied, converted and stored.
//
// Two kinds of wavefront (4 + 4, one of each per SIMD):
//   producer waves issue the direct-to-LDS loads and wait for them (s_waitcnt vmcnt);
//   consumer waves read fragments from LDS, run the matrix instructions and store C.
// The split is what makes the cross-tile overlap possible on this machine: the vector-memory
// counter counts a wave's loads AND its stores, and the two kinds may complete out of order with
// respect to each other, so a wave that has stores of tile t in flight cannot tell when its
// loads of tile t+1 have landed.  Producers never store, consumers never load.
//
// Synchronisation (paper Sec. 4.2 step 5), one block barrier per k-tile i of the stream:
//   producer:  s_waitcnt vmcnt((S-2)*L)  (k-tile i has landed: consumer_wait, first half)
//              s_barrier B_i
//              issue k-tile i+S-1 into slot (i-1) mod S   (producer_acquire: the consumers
//              passed B_i, so they have finished reading k-tile i-1)
//   consumer:  in the last register step of k-tile i-1, after its first matrix instructions
//              (every fragment of k-tile i-1 is in registers by then):
//              s_waitcnt lgkmcnt(0)      (my reads of k-tile i-1 are done: consumer_release)
//              s_barrier B_i             (consumer_wait, second half)
//              then the rest of that step's matrix instructions, which cover the reads of the
//              first fragment of k-tile i: the register-level pipeline is fused across k-tiles
//              (Fig. 3(d)) and across output tiles.  After the last k-tile of a tile comes the
//              epilogue, through an LDS staging area of the wave's own outside the ring.
// Past the end of the stream the producers issue out-of-range loads (they fetch nothing), so the
// number of loads in flight at every wait is the same constant.
//
// The k order per accumulator is the tile-at-a-time kernel's (ko ascending, ki ascending), so
// results are bit-identical to every schedule of that kernel with the same tile.
#pragma once
#include <type_traits>

#include "alcop_kernel.hip.h"

namespace alcop {

// DT, tile, wave tile, stages, layouts as in KCfg; AM: 0 = A is a matrix, 1 = convolution gather
// with one filter tap per k-tile (bk divides the channel count).
// FU: 1 = the consumers' register pipeline is fused across k-tiles and tiles (the barrier sits inside
// the last register step); 0 = it restarts after the barrier that opens each k-tile; 2 = deep:
// three fragments in flight in four register slots, the barrier early in the k-tile (schedules
// name it reg_stages = 4; k-tiles of 64 or 128 only).
template <int DT_, int BM_, int BN_, int BK_, int WM_, int WN_, int S_, int BL_, int AM_, int AL_ = 0,
          int FU_ = 1>
struct SCfg {
  static constexpr int DT = DT_, BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, S = S_;
  static constexpr int BL = BL_, AM = AM_, AL = AL_, FU = FU_;
  static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
  static constexpr int NCW = WAVES_M * WAVES_N;      // consumer waves
  static constexpr int NPW = NCW;                    // producer waves
  static constexpr int NT = (NCW + NPW) * 64, NTP = NPW * 64;
  using OA = Opnd<AL ? LAY_MN : LAY_K, BM, WM, BK, NTP>;
  using OB = Opnd<BL ? LAY_K : LAY_MN, BN, WN, BK, NTP>;
  static constexpr int TM = WM / 32, TN = WN / 32, NKI = BK / 16;
  static constexpr int A_BYTES = OA::BYTES, B_BYTES = OB::BYTES;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int RING_BYTES = S * STAGE_BYTES;
  static constexpr int EPI_WAVE_BYTES = 32 * (WN * 4 + 16);   // staging band of one consumer wave
  static constexpr int LDS_BYTES = RING_BYTES + NCW * EPI_WAVE_BYTES;
  static constexpr int NLA = OA::NL, NLB = OB::NL;
  static constexpr int L = NLA + NLB;                // loads per producer wave and k-tile
  static constexpr int WAIT = (S - 2) * L;
  static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "wave tile");
  static_assert(BK == 32 || BK == 64 || BK == 128, "bk");
  static_assert(S >= 2 && S <= 4, "the stream needs a ring of at least two slots");
  static_assert(AM == 0 || AM == 1, "matrix operand or one-tap-per-k-tile gather");
  static_assert(!(AM != 0 && AL == 1), "the convolution gather produces a K-contiguous A tile");
  static_assert(NCW == 4, "one consumer and one producer wave per SIMD");
  static_assert(WAIT <= 63, "vmcnt is a 6-bit counter");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS ring exceeds 160 KB");
};

template <class C, class HW>
__global__ void __launch_bounds__(C::NT) alcop_stream(const Params p)
{
  constexpr int BM = C::BM, BN = C::BN, BK = C::BK, WM = C::WM, WN = C::WN, S = C::S;
  constexpr int TM = C::TM, TN = C::TN, NKI = C::NKI, NLA = C::NLA, NLB = C::NLB;
  constexpr int STAGE_BYTES = C::STAGE_BYTES, A_BYTES = C::A_BYTES;
  using OA = typename C::OA;
  using OB = typename C::OB;

  const uint32_t lds0 = HW::lds_base();
  const int lane = HW::lane_id();
  const int wave = HW::wave_id();

  // ---- this block's share of the tiles: first, first + grid, first + 2 grid, ... ------------
  const int per_mat = p.ntm * p.ntn;
  const int total = per_mat * p.sbatch;
  const int first = (int)HW::block_x();
  const int my_tiles = (total - first + p.sgrid - 1) / p.sgrid;   // >= 1: the host launches <= total blocks
  const int nko = (p.K + BK - 1) / BK;
  const bool ktail = (p.K % BK) != 0;
  const int T = my_tiles * nko;                                   // k-tiles in this block's stream

  // tile id -> (batch, tm, tn); within a matrix, group_m row tiles form a column-major band so
  // that the tiles the blocks of the chip hold at one time share operand panels in L2
  // Blocks are dealt to the 8 XCDs (each with an L2 of its own) round robin.  When the counts
  // allow, the tile list is permuted so that XCD x owns the x-th eighth of the tile sequence:
  // neighbouring tiles, which share operand panels (and, batched, whole matrices), then meet in
  // one L2 instead of being fetched by all eight.
  const bool by_xcd = p.raster == 1 && (total & 7) == 0 && (p.sgrid & 7) == 0;
  auto decode = [&](int t, int& batch, int& tm, int& tn) __attribute__((always_inline)) {
    if (by_xcd) t = (t & 7) * (total >> 3) + (t >> 3);
    batch = t / per_mat;
    const int r = t - batch * per_mat;
    const int width = p.group_m * p.ntn;
    const int g = r / width;
    const int f = g * p.group_m;
    const int gsz = (p.ntm - f) < p.group_m ? (p.ntm - f) : p.group_m;
    const int rem = r - g * width;
    tm = f + rem % gsz;
    tn = rem / gsz;
  };

  if (wave >= C::NCW) {
    // =============================== producer wave ===========================================
    const int q0 = (wave - C::NCW) * 64 + lane;       // 16-byte LDS slot of this lane in load 0
    const uint32_t wdst = (uint32_t)(wave - C::NCW) * 1024u;
    // producer state of the two operands for the tile being issued, kept in plain variables
    // (descriptor, lane offset of load 0, the bit that pushes a chunk past K out of range in a
    // partial last k-tile, distance between loads, distance between k-tiles)
    typename HW::Rsrc rsA, rsB;
    uint32_t voA = 0, voB = 0, tmA = 0, tmB = 0, stA = 0, stB = 0, ksA = 0, ksB = 0;
    int ih0[NLA], iw0[NLA];
    uint32_t coff[NLA];
    int cs = 0, cc0 = 0, crd = 0, csd = 0;            // filter tap of the next k-tile to issue
    int it = 0, ikt = 0;                              // issue cursor: tile of my list, k-tile in it
    auto open_tile = [&](int j) __attribute__((always_inline)) {
      int batch, tm, tn;
      decode(first + j * p.sgrid, batch, tm, tn);
      const char* Ab = (const char*)p.A + (long)batch * p.strideA * 2;
      const char* Bb = (const char*)p.B + (long)batch * p.strideB * 2;
      if constexpr (C::AM == 0) {
        const LoadState<HW> t = setup_loader<OA, HW>(Ab, tm, p.M, p.lda, p.K, nko, q0);
        rsA = t.rsrc;
        voA = t.voff;
        tmA = t.voff ^ t.voff_t;
        stA = t.step;
        ksA = t.kstep;
      } else {
        rsA = HW::make_rsrc(p.A, (int)p.a_span);
        const int r = q0 / OA::CPR, ph = q0 % OA::CPR;
        const int c = ph ^ OA::template swz<HW>(r);
#pragma unroll
        for (int i = 0; i < NLA; i++) {
          const int m = tm * BM + r + i * OA::RSTEP;
          const int img = m / (p.cP * p.cQ);
          const int pq = m - img * (p.cP * p.cQ);
          const int pp = pq / p.cQ, qq = pq - pp * p.cQ;
          ih0[i] = (m < p.M) ? pp * p.csh - p.cph : -0x40000000;
          iw0[i] = qq * p.csw - p.cpw;
          coff[i] = (uint32_t)((((img * p.cH + (pp * p.csh - p.cph)) * p.cW) + iw0[i]) * p.cC * 2 + c * 16);
        }
        cs = cc0 = crd = csd = 0;
      }
      const LoadState<HW> t = setup_loader<OB, HW>(Bb, tn, p.N, p.ldb, p.K, nko, q0);
      rsB = t.rsrc;
      voB = t.voff;
      tmB = t.voff ^ t.voff_t;
      stB = t.step;
      ksB = t.kstep;
    };
    // the L loads of the next k-tile of the stream (or, past its end, as many loads that fetch
    // nothing) into ring slot `slot`
    auto issue_next = [&](int slot) __attribute__((always_inline)) {
      const uint32_t dst = lds0 + (uint32_t)slot * STAGE_BYTES + wdst;
      const bool live = it < my_tiles;
      const bool tail = ktail && ikt == nko - 1;
      const uint32_t voffA = voA | (tail ? tmA : 0u), voffB = voB | (tail ? tmB : 0u);
      const uint32_t ka = live ? (uint32_t)ikt * ksA : 0x80000000u;
      const uint32_t kb = live ? (uint32_t)ikt * ksB : 0x80000000u;
      const uint32_t tap = (uint32_t)(((crd * p.cW + csd) * p.cC + cc0) * 2);
#pragma unroll
      for (int i = 0; i < NLA; i++) {
        if constexpr (C::AM == 0) {
          HW::dma16(rsA, voffA + ka + (uint32_t)i * stA, dst + i * (C::NPW * 1024));
        } else {
          const bool ok = live && (unsigned)(ih0[i] + crd) < (unsigned)p.cH &&
                          (unsigned)(iw0[i] + csd) < (unsigned)p.cW;
          HW::dma16(rsA, ok ? coff[i] + tap : 0x80000000u, dst + i * (C::NPW * 1024));
        }
      }
#pragma unroll
      for (int i = 0; i < NLB; i++)
        HW::dma16(rsB, voffB + kb + (uint32_t)i * stB, dst + A_BYTES + i * (C::NPW * 1024));
      if (!live) return;
      if constexpr (C::AM == 1) {
        cc0 += BK;
        if (cc0 == p.cC) {
          cc0 = 0; cs++; csd += p.cdw;
          if (cs == p.cS) { cs = 0; csd = 0; crd += p.cdh; }
        }
      }
      if (++ikt == nko) {
        ikt = 0;
        if (++it < my_tiles) open_tile(it);
      }
    };
    open_tile(0);
#pragma unroll
    for (int s = 0; s < S - 1; s++) issue_next(s);
    int wslot = S - 1;
    for (int i = 0; i < T; i++) {
      HW::template wait_vm<C::WAIT>();     // k-tile i of the stream has landed (this wave's part)
      HW::block_barrier();                 // B_i
      issue_next(wslot);                   // into the slot of k-tile i-1, which the consumers left
      wslot = (wslot + 1 == S) ? 0 : wslot + 1;
    }
    HW::template wait_vm<0>();             // the loads that fetch nothing still write LDS: drain them
  } else {
    // =============================== consumer wave ===========================================
    const int wm = wave % C::WAVES_M, wn = wave / C::WAVES_M;
    uint32_t rdA[OA::NRD], rdB[OB::NRD];
    setup_reader<OA, HW>(lane, wm, 0, rdA);
    setup_reader<OB, HW>(lane, wn, A_BYTES, rdB);
    uint32_t curA[OA::NRD], curB[OB::NRD];
    constexpr int NRI = OA::NRI + OB::NRI;
    auto read_one = [&](int ki, int r, u32x4(&fa)[TM], u32x4(&fb)[TN]) __attribute__((always_inline)) {
      if (r < OA::NRI)
        read_instr<OA, HW>(curA, ki, r, fa);
      else
        read_instr<OB, HW>(curB, ki, r - OA::NRI, fb);
    };
    constexpr int NMM = TM * TN;
    constexpr int RPG = (NRI + NMM - 1) / NMM > 2 ? (NRI + NMM - 1) / NMM : 2;   // reads per gap
    const uint32_t ebase = lds0 + C::RING_BYTES + (uint32_t)wave * C::EPI_WAVE_BYTES;
    const bool fused = p.alpha != 1.0f || p.bias != nullptr || p.act != 0;
    auto store_tile = [&](f32x16 (&acc)[TN][TM], int batch, int tm, int tn) __attribute__((always_inline)) {
      // ---- epilogue of a tile (Table 1, epilogue term), overlapped with the producers' loads of
      // the following tiles: convert, transpose one 32-row band at a time through this wave's own
      // staging area, store whole 128-byte lines
      auto epilogue = [&](auto zero) __attribute__((always_inline)) {
        using OT = decltype(zero);
        constexpr int OBY = sizeof(OT);
        constexpr int RS = WN * OBY + 16;
        constexpr int LPR = WN * OBY / 16;
        constexpr int RPI = 64 / LPR;
        typedef OT ot4 __attribute__((ext_vector_type(4)));
        const int m0 = tm * BM + wm * WM, n0 = tn * BN + wn * WN;
        char* Cb = (char*)p.C + (long)batch * p.strideC * OBY;
#pragma unroll
        for (int jj = 0; jj < TM; jj++) {
#pragma unroll
          for (int i = 0; i < TN; i++)
#pragma unroll
            for (int vq = 0; vq < 4; vq++) {
              f32x4 v = {acc[i][jj][4 * vq + 0], acc[i][jj][4 * vq + 1], acc[i][jj][4 * vq + 2],
                         acc[i][jj][4 * vq + 3]};
              if (fused) {
                const int n = n0 + i * 32 + 8 * vq + 4 * (lane >> 5);
                f32x4 bv = {0.f, 0.f, 0.f, 0.f};
                if (p.bias != nullptr && n < p.N) bv = HW::global_load_f32x4(p.bias + n);
#pragma unroll
                for (int e = 0; e < 4; e++) {
                  float t = v[e] * p.alpha + bv[e];
                  v[e] = (p.act == 1 && t < 0.f) ? 0.f : t;
                }
              }
              const ot4 h = {HW::template cvt<OT>(v[0]), HW::template cvt<OT>(v[1]),
                             HW::template cvt<OT>(v[2]), HW::template cvt<OT>(v[3])};
              HW::lds_write(ebase + (lane & 31) * RS + (i * 32 + 8 * vq + 4 * (lane >> 5)) * OBY, h);
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
              if (!lane_ok) r = 0;        // every lane takes part in the read; idle ones store nothing
            }
            const u32x4 v = HW::lds_read16(ebase + r * RS + c16 * 16);
            const int m = m0 + jj * 32 + r;
            const int n = n0 + c16 * (16 / OBY);
            if (lane_ok && m < p.M && n < p.N) HW::global_store16(Cb + ((long)m * p.ldc + n) * OBY, v);
          }
        }
      };
      if (p.out_dtype == 2)
        epilogue(0.0f);
      else if (p.out_dtype == 0)
        epilogue((_Float16)0);
      else
        epilogue((__bf16)0);
    };
    int slot = 0;
    int i_stream = 0;                      // k-tile of the stream being consumed
    u32x4 fa[2][TM], fb[2][TN];
    auto open_slot = [&]() __attribute__((always_inline)) {
      const uint32_t sbase = lds0 + (uint32_t)slot * STAGE_BYTES;
      slot = (slot + 1 == S) ? 0 : slot + 1;
#pragma unroll
      for (int i = 0; i < OA::NRD; i++) curA[i] = sbase + rdA[i];
#pragma unroll
      for (int i = 0; i < OB::NRD; i++) curB[i] = sbase + rdB[i];
    };
    if constexpr (C::FU == 2) {
      // Deep register pipeline: D = 3 fragments are in flight ahead of the one the matrix
      // instructions consume, in R = 4 rotating register slots (a k-tile has 4 or 8 fragments, so
      // fragment ki always lives in slot ki % 4 and every register index is a compile-time
      // constant).  In step ki the fragment 3 steps ahead is read: (i, 3) in step 0, then
      // (i+1, 0), (i+1, 1), ... of the NEXT k-tile.  The barrier B_{i+1} therefore stands between
      // steps 0 and 1 of k-tile i; when a wave passes it, the fragments of the next three steps
      // are already in registers, so no matrix instruction behind the barrier waits for LDS.
      constexpr int R = 4, D = 3;
      static_assert(NKI % R == 0, "the deep consumer needs a k-tile of 64 or 128");
      u32x4 ga[R][TM], gb[R][TN];
      int j = 0, ko = 0, batch, tm, tn;
      decode(first, batch, tm, tn);
      f32x16 acc[TN][TM];
#pragma unroll
      for (int a = 0; a < TN; a++)
#pragma unroll
        for (int b = 0; b < TM; b++)
#pragma unroll
          for (int v = 0; v < 16; v++) acc[a][b][v] = 0.f;
      HW::wait_lds();
      HW::block_barrier();                 // B_0: k-tile 0 has landed for every producer wave
      open_slot();
#pragma unroll
      for (int ki = 0; ki < D; ki++)
#pragma unroll
        for (int r = 0; r < NRI; r++) read_one(ki, r, ga[ki], gb[ki]);
      HW::sched_fence();
      constexpr int RPM = (NRI + NMM - 1) / NMM > 2 ? (NRI + NMM - 1) / NMM : 2;   // reads per matrix instruction
      for (int i = 0; i < T; i++) {
        const bool more = i + 1 < T;       // another k-tile follows in the stream (uniform)
#pragma unroll
        for (int ki = 0; ki < NKI; ki++) {
          // the fragment read during this step: (i, ki + D) while that is inside this k-tile,
          // else (i + 1, ki + D - NKI), for which B_{i+1} must have been passed
          const bool next_tile = ki + D >= NKI;
          if (ki + D == NKI && more) {
            // every fragment of k-tile i has been read (the last one during the step before)
            HW::wait_lds();                // consumer_release: my reads of k-tile i are done
            HW::block_barrier();           // B_{i+1}: k-tile i+1 has landed, slot i may be refilled
            open_slot();
            HW::sched_fence();
          }
          const int kr = next_tile ? ki + D - NKI : ki + D;     // fragment index within its k-tile
#pragma unroll
          for (int m = 0; m < NMM; m++) {
            const int a = m / TM, b = m % TM;
            acc[a][b] = HW::template mma<C::DT>(gb[ki % R][a], ga[ki % R][b], acc[a][b]);
            if (!next_tile || more) {
#pragma unroll
              for (int r = m * RPM; r < (m + 1) * RPM && r < NRI; r++)
                read_one(kr, r, ga[(ki + D) % R], gb[(ki + D) % R]);
            }
            HW::sched_fence();
          }
        }
        if (++ko == nko) {
          store_tile(acc, batch, tm, tn);
          ko = 0;
          if (++j < my_tiles) decode(first + j * p.sgrid, batch, tm, tn);
#pragma unroll
          for (int a = 0; a < TN; a++)
#pragma unroll
            for (int b = 0; b < TM; b++)
#pragma unroll
              for (int v = 0; v < 16; v++) acc[a][b][v] = 0.f;
        }
      }
      HW::wait_lds();
      return;
    }
    // The register-level pipeline runs across k-tiles and across output tiles (Fig. 3(d)): the
    // barrier B_{i+1} sits after the first matrix instructions of the LAST step of k-tile i, when
    // every fragment of k-tile i is already in registers, and the rest of that step's matrix
    // instructions cover the reads of the first fragment of k-tile i+1.
    if constexpr (C::FU) {
      HW::wait_lds();
      HW::block_barrier();                 // B_0: k-tile 0 has landed for every producer wave
      open_slot();
#pragma unroll
      for (int r = 0; r < NRI; r++) read_one(0, r, fa[0], fb[0]);
      HW::sched_fence();
    }
    static_assert(NKI % 2 == 0, "fragment parity must repeat per k-tile");
    constexpr int FIRST = NMM >= 8 ? NMM / 4 : 1;
    constexpr int GAPS = NMM - FIRST > 0 ? NMM - FIRST : 1;
    constexpr int RPGL = (NRI + GAPS - 1) / GAPS > 2 ? (NRI + GAPS - 1) / GAPS : 2;   // reads per gap, last step
    for (int j = 0; j < my_tiles; j++) {
      int batch, tm, tn;
      decode(first + j * p.sgrid, batch, tm, tn);
      f32x16 acc[TN][TM];
#pragma unroll
      for (int a = 0; a < TN; a++)
#pragma unroll
        for (int b = 0; b < TM; b++)
#pragma unroll
          for (int v = 0; v < 16; v++) acc[a][b][v] = 0.f;
      for (int ko = 0; ko < nko; ko++) {
        const bool more = C::FU && i_stream + 1 < T;   // another k-tile follows in the stream (uniform)
        i_stream++;
        if constexpr (!C::FU) {
          HW::wait_lds();                  // consumer_release: my reads of the previous k-tile are done
          HW::block_barrier();             // B_i: k-tile i has landed for every producer wave
          open_slot();
#pragma unroll
          for (int r = 0; r < NRI; r++) read_one(0, r, fa[0], fb[0]);
          HW::sched_fence();
        }
#pragma unroll
        for (int ki = 0; ki < NKI; ki++) {
#pragma unroll
          for (int m = 0; m < NMM; m++) {
            const int a = m / TM, b = m % TM;
            acc[a][b] = HW::template mma<C::DT>(fb[ki & 1][a], fa[ki & 1][b], acc[a][b]);
            if (ki + 1 < NKI) {
              // reads of fragment ki+1, spread over the matrix instructions of fragment ki
#pragma unroll
              for (int r = m * RPG; r < (m + 1) * RPG && r < NRI; r++)
                read_one(ki + 1, r, fa[(ki + 1) & 1], fb[(ki + 1) & 1]);
            } else if (more) {
              if (m + 1 == FIRST || (FIRST >= NMM && m == NMM - 1)) {
                HW::wait_lds();            // consumer_release: my reads of k-tile i are done
                HW::block_barrier();       // B_{i+1}: k-tile i+1 has landed, slot i may be refilled
                open_slot();
              }
              if (m >= FIRST || m == NMM - 1) {
                const int g = m >= FIRST ? m - FIRST : 0;
                const int r1 = (m == NMM - 1) ? NRI : (g + 1) * RPGL;   // the last gap takes what is left
#pragma unroll
                for (int r = g * RPGL; r < r1 && r < NRI; r++) read_one(0, r, fa[0], fb[0]);
              }
            }
            HW::sched_fence();
          }
        }
      }
      store_tile(acc, batch, tm, tn);
    }
    HW::wait_lds();
  }
}

}  // namespace alcop
