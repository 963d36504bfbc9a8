// Functional model of the hardware operations the pipelined main loop is written against,
// for running the kernel template itself on the CPU (test infrastructure, never part of the
// product library).
//
// How it runs a block.  Every lane of the block is a fibre (ucontext) that executes the kernel
// function as ordinary C++.  Operations that exchange data between the lanes of a wavefront (the
// matrix instruction, the transposing LDS read, and LDS traffic in general: one lane may read
// what another lane of its wave wrote one instruction earlier) make the lane yield until all 64
// lanes of its wave have arrived; the block barrier does the same over all lanes.
// A scheduler resumes runnable lanes, always preferring one wave (the first or the last, by
// policy), so that wave runs as far ahead of the others as the kernel's synchronisation allows.
//
// What it checks.
//   * every LDS access lies inside the block's dynamic LDS and is naturally aligned;
//   * every global access lies inside a buffer the test registered: stores, bias reads, L2
//     touches, and the bytes a buffer descriptor admits (a direct-to-LDS load inside
//     num_records must also be inside the operand);
//   * descriptor words and LDS destinations of direct-to-LDS loads are the same in all lanes
//     of a wave (on the machine they live in scalar registers);
//   * the wait counters: with late landing, a direct-to-LDS load poisons its destination when
//     it is issued (the slot's content is undefined while the load is in flight) and delivers
//     its data only when a later s_waitcnt vmcnt(N) of the same lane forces it to; with early
//     landing it delivers at once.  A read that the kernel's waits and barriers do not order
//     after the landing, or before the refill, then returns poison (NaN patterns) or the wrong
//     k-tile, and the result differs from the oracle's;
//   * the release of a ring slot: an LDS read counts as in flight from its issue until the
//     lane's next s_waitcnt lgkmcnt(0) (the compiler's own waits before a register is used are
//     not visible here, so this is the conservative reading); a direct-to-LDS load issued onto
//     bytes that any lane may still be reading is an error;
//   * no load is in flight and no lane is waiting when the kernel returns.
//
// The semantics modelled here were established by probing an MI355X:
//   buffer_load_dwordx4 ... lds: lane l's 16 bytes land at M0 + 16*l; an offset at or beyond
//     num_records delivers zeros;
//   ds_read_b64_tr_b16: in each group of 16 lanes, lane i receives as element e the 16-bit
//     element i%4 of the 8 bytes addressed by lane 4e + i/4;
//   v_mfma_f32_32x32x16: X lane l = row l%32, k = 8*(l/32)..+7; Y lane l = column l%32, same
//     k; D lane l = column l%32, rows 8*(v/4) + 4*(l/32) + v%4, v = 0..15.
#pragma once
#include <stdint.h>
#include <string.h>
#include <sys/mman.h>
#include <ucontext.h>

#include <cstdarg>
#include <cstdio>
#include <deque>
#include <string>
#include <vector>

#include "alcop_kernel.hip.h"
#include "alcop_stream.hip.h"

namespace emu {

using alcop::f32x16;
using alcop::f32x4;
using alcop::u32x2;
using alcop::u32x4;

// ---- configuration and error log ----------------------------------------------------------
struct Buffer {
  const char* ptr;
  size_t bytes;
  bool writable;
};
struct Config {
  std::vector<Buffer> buffers;
  bool late_landing = true;    // direct-to-LDS data lands only when a wait forces it
  bool last_wave_first = false;
  int mutation = 0;            // a planted synchronisation mistake (see emu_set_mutation)
  bool any_address = false;    // no operand ranges declared: global accesses are not checked
  std::vector<std::string> errors;
  long n_errors = 0;
};
inline Config& cfg()
{
  static Config c;
  return c;
}
inline void fail(const char* fmt, ...) __attribute__((format(printf, 1, 2)));
inline void fail(const char* fmt, ...)
{
  Config& c = cfg();
  c.n_errors++;
  if (c.errors.size() >= 32) return;
  char buf[256];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  c.errors.push_back(buf);
}
inline bool in_buffer(const void* p, size_t n, bool write)
{
  const char* a = (const char*)p;
  if (cfg().any_address) return true;
  for (const Buffer& b : cfg().buffers)
    if (a >= b.ptr && a + n <= b.ptr + b.bytes && (!write || b.writable)) return true;
  return false;
}

// ---- block state ----------------------------------------------------------------------------
constexpr uint32_t LDS_BASE = 1024;   // a non-zero, 1024-aligned base: a missing base shows up
constexpr uint16_t POISON16 = 0x7fff; // NaN as fp16 and as bf16

struct Pending {
  uint32_t dst;
  uint32_t bytes;          // 16 (tile load) or 4 (L2 touch)
  unsigned char data[16];
};
enum { RUN = 0, WAIT_WAVE = 1, WAIT_BLOCK = 2, DONE = 3 };
struct Lane {
  ucontext_t ctx;
  int state = RUN;
  int mma_par = 0, tr_par = 0;
  long n_rsrc = 0, n_dma = 0;      // per-lane operation counters for the uniformity checks
  std::deque<Pending> pending;
  std::vector<std::pair<uint32_t, uint32_t>> reads;   // LDS reads since the last lgkmcnt(0) wait
};
struct Wave {
  int arrived = 0, runnable = 0;
  u32x4 X[2][64], Y[2][64];
  uint32_t T[2][64];
  std::vector<uint64_t> rsrc_log;  // (base ^ bytes) of make_rsrc call #k, as lane 0..63 see it
  std::vector<uint32_t> dma_log;   // LDS destination of direct-to-LDS load #k
};
struct Block {
  int nt = 0, nwaves = 0;
  uint32_t bx = 0, by = 0, bz = 0;
  std::vector<unsigned char> lds;  // LDS_BASE + lds_bytes
  std::vector<uint16_t> reading;   // per LDS byte: reads that may still be in flight
  uint32_t lds_bytes = 0;
  std::vector<Lane> lanes;
  std::vector<Wave> waves;
  int block_arrived = 0, done = 0;
  int cur = 0;
  ucontext_t sched;
  void (*entry)(const void*) = nullptr;   // the kernel, applied to its parameter struct
  const void* params = nullptr;
};
inline Block*& blk()
{
  static Block* b = nullptr;
  return b;
}

inline void yield_to_scheduler()
{
  Block& b = *blk();
  swapcontext(&b.lanes[b.cur].ctx, &b.sched);
}
inline void wave_sync()
{
  Block& b = *blk();
  const int me = b.cur, w = me >> 6;
  Wave& W = b.waves[w];
  if (++W.arrived == 64) {
    W.arrived = 0;
    for (int l = w * 64; l < w * 64 + 64; l++)
      if (b.lanes[l].state == WAIT_WAVE) {
        b.lanes[l].state = RUN;
        W.runnable++;
      }
    return;
  }
  b.lanes[me].state = WAIT_WAVE;
  W.runnable--;
  yield_to_scheduler();
}
inline void block_sync()
{
  Block& b = *blk();
  const int me = b.cur;
  if (++b.block_arrived == b.nt) {
    b.block_arrived = 0;
    for (int l = 0; l < b.nt; l++)
      if (b.lanes[l].state == WAIT_BLOCK) {
        b.lanes[l].state = RUN;
        b.waves[l >> 6].runnable++;
      }
    return;
  }
  b.lanes[me].state = WAIT_BLOCK;
  b.waves[me >> 6].runnable--;
  yield_to_scheduler();
}

inline unsigned char* lds_ptr(uint32_t addr, uint32_t n, uint32_t align, const char* what)
{
  Block& b = *blk();
  if (addr < LDS_BASE || addr + n > LDS_BASE + b.lds_bytes || addr + n < addr) {
    fail("%s: LDS access [%u, +%u) outside the block's %u bytes (block %u,%u thread %d)", what,
         addr - LDS_BASE, n, b.lds_bytes, b.bx, b.by, b.cur);
    return nullptr;
  }
  if (addr % align) {
    fail("%s: LDS address %u not aligned to %u (thread %d)", what, addr - LDS_BASE, align, b.cur);
    return nullptr;
  }
  return b.lds.data() + addr;
}
// An LDS read of [addr, addr + n) by the current lane stays "in flight" until its next wait.
inline void note_read(uint32_t addr, uint32_t n)
{
  Block& b = *blk();
  for (uint32_t i = 0; i < n; i++) b.reading[addr + i]++;
  b.lanes[b.cur].reads.emplace_back(addr, n);
}
inline void reads_done()
{
  Block& b = *blk();
  for (const auto& r : b.lanes[b.cur].reads)
    for (uint32_t i = 0; i < r.second; i++) b.reading[r.first + i]--;
  b.lanes[b.cur].reads.clear();
}
inline void land(const Pending& p)
{
  if (unsigned char* d = lds_ptr(p.dst, p.bytes, 4, "direct-to-LDS landing")) memcpy(d, p.data, p.bytes);
}

inline float f16_to_float(uint16_t h)
{
  const uint32_t s = (uint32_t)(h >> 15) << 31, e = (h >> 10) & 31, m = h & 1023;
  uint32_t u;
  if (e == 0) {
    if (m == 0) {
      u = s;
    } else {   // subnormal: value = m * 2^-24
      float f = (float)m * 5.9604644775390625e-8f;
      memcpy(&u, &f, 4);
      u |= s;
    }
  } else if (e == 31) {
    u = s | 0x7f800000u | (m << 13);
  } else {
    u = s | ((e + 112) << 23) | (m << 13);
  }
  float f;
  memcpy(&f, &u, 4);
  return f;
}
inline float bf16_to_float(uint16_t h)
{
  const uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}
// round to nearest even, fp32 -> fp16 bits
inline uint16_t float_to_f16(float f)
{
  uint32_t u;
  memcpy(&u, &f, 4);
  const uint32_t s = (u >> 16) & 0x8000u;
  const uint32_t a = u & 0x7fffffffu;
  if (a >= 0x7f800000u) return (uint16_t)(s | 0x7c00u | (a > 0x7f800000u ? 0x200u : 0));
  if (a >= 0x477ff000u) return (uint16_t)(s | 0x7c00u);          // rounds to infinity
  if (a < 0x33000001u) return (uint16_t)s;                        // rounds to zero
  int e = (int)(a >> 23) - 127;
  uint32_t m = (a & 0x7fffffu) | 0x800000u;                        // 24-bit significand
  int shift = e >= -14 ? 13 : 13 + (-14 - e);                      // bits dropped
  uint32_t q = m >> shift, rem = m & ((1u << shift) - 1), half = 1u << (shift - 1);
  if (rem > half || (rem == half && (q & 1))) q++;
  uint32_t out = e >= -14 ? ((uint32_t)(e + 15 - 1) << 10) + q : q;   // q carries the hidden bit
  return (uint16_t)(s | out);
}
inline uint16_t float_to_bf16(float f)
{
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1);
  return (uint16_t)(u >> 16);
}

// ---- the policy class -------------------------------------------------------------------------
struct Rsrc {
  const char* base;
  uint32_t bytes;
};

struct Emu {
  static constexpr bool kSwizzle = true;
  using Rsrc = emu::Rsrc;

  static int lane_id() { return blk()->cur & 63; }
  static int wave_id() { return blk()->cur >> 6; }
  static uint32_t block_x() { return blk()->bx; }
  static uint32_t block_y() { return blk()->by; }
  static uint32_t block_z() { return blk()->bz; }
  static uint32_t lds_base() { return LDS_BASE; }

  static Rsrc make_rsrc(const void* base, int bytes)
  {
    Block& b = *blk();
    Lane& L = b.lanes[b.cur];
    Wave& W = b.waves[b.cur >> 6];
    const uint64_t sig = (uint64_t)(uintptr_t)base ^ ((uint64_t)(uint32_t)bytes << 48);
    const size_t k = (size_t)L.n_rsrc++;
    if (k == W.rsrc_log.size())
      W.rsrc_log.push_back(sig);
    else if (W.rsrc_log[k] != sig)
      fail("buffer descriptor #%zu differs between lanes of wave %d (thread %d)", k, b.cur >> 6, b.cur);
    if (bytes < 0) fail("buffer descriptor with negative size %d (thread %d)", bytes, b.cur);
    return Rsrc{(const char*)base, (uint32_t)bytes};
  }

  static void deliver(uint32_t dst, uint32_t n, const unsigned char* data)
  {
    Block& b = *blk();
    Pending p;
    p.dst = dst;
    p.bytes = n;
    memcpy(p.data, data, n);
    if (lds_ptr(dst, n, 4, "direct-to-LDS destination"))
      for (uint32_t i = 0; i < n; i++)
        if (b.reading[dst + i]) {
          fail("direct-to-LDS load onto LDS bytes %u.. that a read issued before the last "
               "lgkmcnt(0) wait may still be fetching (block %u,%u thread %d)",
               dst + i - LDS_BASE, b.bx, b.by, b.cur);
          break;
        }
    if (!cfg().late_landing) {
      land(p);
      return;
    }
    // in flight: the destination's content is undefined until the load lands
    if (unsigned char* d = lds_ptr(dst, n, 4, "direct-to-LDS destination"))
      for (uint32_t i = 0; i + 1 < n; i += 2) memcpy(d + i, &POISON16, 2);
    b.lanes[b.cur].pending.push_back(p);
  }

  static void dma16(Rsrc r, uint32_t voff, uint32_t lds_dst)
  {
    Block& b = *blk();
    Lane& L = b.lanes[b.cur];
    Wave& W = b.waves[b.cur >> 6];
    const size_t k = (size_t)L.n_dma++;
    if (k == W.dma_log.size())
      W.dma_log.push_back(lds_dst);
    else if (W.dma_log[k] != lds_dst)
      fail("LDS destination of direct-to-LDS load #%zu differs between lanes of wave %d", k, b.cur >> 6);
    if (lds_dst % 16) fail("direct-to-LDS destination %u not a multiple of 16", lds_dst);
    unsigned char data[16] = {0};
    if ((uint64_t)voff + 16 <= r.bytes) {
      if (voff % 16) fail("direct-to-LDS source offset %u not a multiple of 16 (thread %d)", voff, b.cur);
      if (in_buffer(r.base + voff, 16, false))
        memcpy(data, r.base + voff, 16);
      else
        fail("descriptor admits offset %u (num_records %u) but the bytes lie outside every operand "
             "(block %u,%u thread %d)", voff, r.bytes, b.bx, b.by, b.cur);
    } else if (voff < r.bytes) {
      fail("direct-to-LDS load straddles num_records: offset %u, num_records %u", voff, r.bytes);
    }
    deliver(lds_dst + 16u * (uint32_t)(b.cur & 63), 16, data);
  }

  static void touch4(const char* gptr, uint32_t lds_dst)
  {
    Block& b = *blk();
    Lane& L = b.lanes[b.cur];
    Wave& W = b.waves[b.cur >> 6];
    const size_t k = (size_t)L.n_dma++;
    if (k == W.dma_log.size())
      W.dma_log.push_back(lds_dst);
    else if (W.dma_log[k] != lds_dst)
      fail("LDS destination of L2 touch #%zu differs between lanes of wave %d", k, b.cur >> 6);
    unsigned char data[4] = {0};
    if ((uintptr_t)gptr % 4) fail("L2 touch address not 4-byte aligned (thread %d)", b.cur);
    if (in_buffer(gptr, 4, false))
      memcpy(data, gptr, 4);
    else
      fail("L2 touch outside every operand: block %u,%u thread %d", b.bx, b.by, b.cur);
    deliver(lds_dst + 4u * (uint32_t)(b.cur & 63), 4, data);
  }

  template <int N>
  static void wait_vm()
  {
    Block& b = *blk();
    std::deque<Pending>& q = b.lanes[b.cur].pending;
    const int mut = cfg().mutation;
    if (mut == 3 && N != 0) return;
    const int allowed = (mut == 1 && N != 0) ? N + 2 : N;
    while ((int)q.size() > allowed) {   // loads return in issue order
      land(q.front());
      q.pop_front();
    }
  }
  static void wait_lds()           // reads deliver at once here; the wait ends their "in flight" mark
  {
    if (cfg().mutation == 4) return;
    reads_done();
  }
  static void block_barrier()
  {
    if (cfg().mutation == 2) return;
    block_sync();
  }
  static void sched_fence() {}

  template <int DT>
  static f32x16 mma(u32x4 x, u32x4 y, f32x16 acc)
  {
    Block& b = *blk();
    const int l = b.cur & 63;
    Lane& L = b.lanes[b.cur];
    Wave& W = b.waves[b.cur >> 6];
    const int par = L.mma_par;
    L.mma_par ^= 1;
    W.X[par][l] = x;
    W.Y[par][l] = y;
    wave_sync();
    const int j = l & 31;
    for (int v = 0; v < 16; v++) {
      const int i = 8 * (v / 4) + 4 * (l >> 5) + (v & 3);
      float s = acc[v];
      for (int k = 0; k < 16; k++) {
        const u32x4 xr = W.X[par][i + 32 * (k >> 3)], yr = W.Y[par][j + 32 * (k >> 3)];
        const int e = k & 7;
        const uint16_t xb = (uint16_t)(xr[e >> 1] >> (16 * (e & 1)));
        const uint16_t yb = (uint16_t)(yr[e >> 1] >> (16 * (e & 1)));
        const float xf = DT == 0 ? f16_to_float(xb) : bf16_to_float(xb);
        const float yf = DT == 0 ? f16_to_float(yb) : bf16_to_float(yb);
        s += xf * yf;
      }
      acc[v] = s;
    }
    return acc;
  }

  // The lanes of a wave execute an instruction together, so an LDS instruction sees every LDS
  // write the wave's earlier instructions made, in all lanes: each LDS read or write of the
  // model starts by waiting for the other lanes of the wave.
  static u32x4 lds_read16(uint32_t addr)
  {
    wave_sync();
    u32x4 v = {0, 0, 0, 0};
    if (const unsigned char* p = lds_ptr(addr, 16, 16, "ds_read_b128")) {
      memcpy(&v, p, 16);
      note_read(addr, 16);
    }
    return v;
  }
  static u32x2 lds_read_tr8(uint32_t addr)
  {
    Block& b = *blk();
    const int l = b.cur & 63;
    Lane& L = b.lanes[b.cur];
    Wave& W = b.waves[b.cur >> 6];
    const int par = L.tr_par;
    L.tr_par ^= 1;
    W.T[par][l] = addr;
    wave_sync();
    const int g = l & ~15, i = l & 15;
    uint16_t out[4] = {0, 0, 0, 0};
    for (int e = 0; e < 4; e++) {
      const uint32_t a = W.T[par][g + 4 * e + i / 4];
      if (const unsigned char* p = lds_ptr(a, 8, 8, "ds_read_b64_tr_b16")) {
        memcpy(&out[e], p + 2 * (i % 4), 2);
        note_read(a + 2 * (i % 4), 2);
      }
    }
    u32x2 v;
    memcpy(&v, out, 8);
    return v;
  }
  template <class V>
  static void lds_write(uint32_t addr, V v)
  {
    wave_sync();
    if (unsigned char* p = lds_ptr(addr, sizeof(V), sizeof(V), "ds_write")) memcpy(p, &v, sizeof(V));
  }

  static void global_store16(void* ptr, u32x4 v)
  {
    Block& b = *blk();
    if ((uintptr_t)ptr % 16) fail("16-byte global store to an unaligned address (thread %d)", b.cur);
    if (in_buffer(ptr, 16, true))
      memcpy(ptr, &v, 16);
    else
      fail("global store outside the output: block %u,%u thread %d", b.bx, b.by, b.cur);
  }
  static f32x4 global_load_f32x4(const float* ptr)
  {
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if ((uintptr_t)ptr % 16) fail("16-byte global load from an unaligned address (thread %d)", blk()->cur);
    if (in_buffer(ptr, 16, false))
      memcpy(&v, ptr, 16);
    else
      fail("global load outside every operand (thread %d)", blk()->cur);
    return v;
  }
  template <class T>
  static T global_load_elem(const void* ptr)
  {
    T v = 0;
    if ((uintptr_t)ptr % sizeof(T)) fail("element load from a misaligned address (thread %d)", blk()->cur);
    if (in_buffer(ptr, sizeof(T), false))
      memcpy(&v, ptr, sizeof(T));
    else
      fail("element load outside every operand: block %u,%u thread %d", blk()->bx, blk()->by, blk()->cur);
    return v;
  }
  template <class T>
  static void global_store_elem(void* ptr, T v)
  {
    if ((uintptr_t)ptr % sizeof(T)) fail("element store to a misaligned address (thread %d)", blk()->cur);
    if (in_buffer(ptr, sizeof(T), true))
      memcpy(ptr, &v, sizeof(T));
    else
      fail("element store outside the output: block %u,%u thread %d", blk()->bx, blk()->by, blk()->cur);
  }
  static uint16_t global_load_u16(const void* ptr) { return global_load_elem<uint16_t>(ptr); }
  static uint32_t global_load_u32(const void* ptr) { return global_load_elem<uint32_t>(ptr); }
  static void global_store_u16(void* ptr, uint16_t v) { global_store_elem<uint16_t>(ptr, v); }
  static void global_store_u32(void* ptr, uint32_t v) { global_store_elem<uint32_t>(ptr, v); }
  template <class OT>
  static OT cvt(float v)
  {
    if constexpr (sizeof(OT) == 4) {
      return v;
    } else {
      const uint16_t bits = __is_same(OT, _Float16) ? float_to_f16(v) : float_to_bf16(v);
      OT o;
      memcpy(&o, &bits, 2);
      return o;
    }
  }
};

// ---- running a grid -----------------------------------------------------------------------------
constexpr size_t STACK_BYTES = 256 * 1024;

inline void lane_main()
{
  Block& b = *blk();
  const int me = b.cur;
  b.entry(b.params);
  // the lane has left the kernel
  b.cur = me;
  if (!b.lanes[me].pending.empty())
    fail("thread %d returned with %zu loads in flight", me, b.lanes[me].pending.size());
  b.lanes[me].state = DONE;
  b.waves[me >> 6].runnable--;
  b.done++;
}

inline void run_block(Block& b)
{
  blk() = &b;
  char* stacks = (char*)mmap(nullptr, STACK_BYTES * b.nt, PROT_READ | PROT_WRITE,
                             MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE, -1, 0);
  if (stacks == (char*)MAP_FAILED) {
    fail("mmap of the lane stacks failed");
    return;
  }
  for (int l = 0; l < b.nt; l++) {
    getcontext(&b.lanes[l].ctx);
    b.lanes[l].ctx.uc_stack.ss_sp = stacks + STACK_BYTES * l;
    b.lanes[l].ctx.uc_stack.ss_size = STACK_BYTES;
    b.lanes[l].ctx.uc_link = &b.sched;
    makecontext(&b.lanes[l].ctx, (void (*)())lane_main, 0);
  }
  for (Wave& w : b.waves) w.runnable = 64;
  const bool rev = cfg().last_wave_first;
  while (b.done < b.nt) {
    int w = -1;
    for (int k = 0; k < b.nwaves; k++) {
      const int c = rev ? b.nwaves - 1 - k : k;
      if (b.waves[c].runnable > 0) {
        w = c;
        break;
      }
    }
    if (w < 0) {
      fail("deadlock: block %u,%u has %d lanes left, none runnable (a barrier some lanes never reach)",
           b.bx, b.by, b.nt - b.done);
      break;
    }
    for (int l = w * 64; l < w * 64 + 64; l++)
      if (b.lanes[l].state == RUN) {
        b.cur = l;
        swapcontext(&b.sched, &b.lanes[l].ctx);
      }
  }
  munmap(stacks, STACK_BYTES * b.nt);
  blk() = nullptr;
}

// Runs a whole grid, block after block (threads per block a multiple of 64).  Returns the
// number of errors logged so far.
inline long run_grid(void (*entry)(const void*), const void* params, int threads, uint32_t lds_bytes,
                     unsigned gx, unsigned gy, unsigned gz)
{
  for (unsigned bz = 0; bz < gz; bz++)
    for (unsigned by = 0; by < gy; by++)
      for (unsigned bx = 0; bx < gx; bx++) {
        Block b;
        b.nt = threads;
        b.nwaves = threads / 64;
        b.bx = bx;
        b.by = by;
        b.bz = bz;
        b.lds_bytes = lds_bytes;
        b.lds.assign(LDS_BASE + lds_bytes, 0);
        b.reading.assign(LDS_BASE + lds_bytes, 0);
        for (size_t i = 0; i + 1 < b.lds.size(); i += 2) memcpy(b.lds.data() + i, &POISON16, 2);
        b.lanes.resize(threads);
        b.waves.resize(threads / 64);
        b.entry = entry;
        b.params = params;
        run_block(b);
        if (cfg().n_errors > 1000) return cfg().n_errors;
      }
  return cfg().n_errors;
}

template <class C>
void mainloop_entry(const void* p)
{
  alcop::alcop_mainloop<C, Emu>(*(const alcop::Params*)p);
}
template <class C>
void stream_entry(const void* p)
{
  alcop::alcop_stream<C, Emu>(*(const alcop::Params*)p);
}

}  // namespace emu
