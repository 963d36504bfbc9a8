// C ABI of the library: argument validation, schedule lookup, launch, timing and the
// model-ranked tuner.  Declarations and argument contracts are in include/alcop.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <tuple>
#include <vector>

#include "../../include/alcop.h"
#include "alcop_model.h"
#include "alcop_registry.h"

namespace alcop {

const std::vector<KernelEntry>& registry()
{
  static const std::vector<KernelEntry> table = [] {
    std::vector<KernelEntry> t;
    register_f16_kn_big(t);
    register_f16_kn_mid(t);
    register_f16_kn_small(t);
    register_bf16_kn(t);
    register_nk(t);
    register_conv(t);
    register_ta(t);
    register_conv_krsc(t);
    register_conv_anyc(t);
    register_conv_patch(t);
    register_bk128(t);
    register_deep(t);
    register_wide(t);
    register_pf(t);
    register_stream(t);
    register_splitk_gemm(t);
    register_splitk_conv(t);
    return t;
  }();
  return table;
}

namespace {

struct Call {
  alcop_op op;
  const void *A, *B;
  void* C;
  int batch, M, N, K;
  long lda, ldb, ldc, strideA, strideB, strideC;
  int transA, transB;
  alcop_dtype in, out;
  // conv geometry
  int cN, cH, cW, cC, cK, cR, cS, csh, csw, cph, cpw, cP, cQ;
  int cdh, cdw;   // dilation
  // fused epilogue
  float alpha;
  const void* bias;
  int act;
};

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

alcop_problem problem_of(const Call& c)
{
  alcop_problem p;
  p.op = c.op;
  p.batch = c.batch;
  p.M = c.M;
  p.N = c.N;
  p.K = c.K;
  p.transB = c.transB;
  p.transA = c.transA;
  p.in = c.in;
  p.out = c.out;
  p.conv_C = c.op == ALCOP_OP_CONV2D ? c.cC : 0;
  return p;
}

// Loader of the A operand a problem needs with k-tile bk: 0 = matrix; 1 = convolution gather
// whose k-tiles lie inside one filter tap (bk divides the channel count); 2 = gather for any
// channel count that is a multiple of 8.
// 3 = schedule variant 1 of a convolution: the input patch stays in LDS (bk equals the channel count).
int a_mode(const alcop_problem& p, int bk, int variant)
{
  if (p.op != ALCOP_OP_CONV2D) return 0;
  if (variant == 1) return 3;
  return (bk > 0 && p.conv_C % bk == 0) ? 1 : 2;
}

const KernelEntry* find_entry(const alcop_problem& p, const alcop_sched& s, int sk)
{
  const int am = a_mode(p, s.bk, s.variant);
  for (const KernelEntry& e : registry())
    if (e.sk == sk && e.dt == (int)p.in && e.bl == (p.transB ? 1 : 0) && e.al == (p.transA ? 1 : 0) &&
        e.am == am && e.bm == s.bm &&
        e.bn == s.bn && e.bk == s.bk && e.wm == s.wm && e.wn == s.wn && e.stages == s.stages &&
        e.reg_stages == s.reg_stages && e.fuse == (s.fuse_inner ? 1 : 0) &&
        e.pf == (s.l2_prefetch > 0 ? 1 : 0) && e.st == (s.variant == 2 ? 1 : 0))
      return &e;
  return nullptr;
}

int check_problem(const alcop_problem& p)
{
  if (p.in != ALCOP_F16 && p.in != ALCOP_BF16) return ALCOP_ERR_DTYPE;
  if (p.out != ALCOP_F16 && p.out != ALCOP_BF16 && p.out != ALCOP_F32) return ALCOP_ERR_DTYPE;
  if (p.op != ALCOP_OP_GEMM && p.op != ALCOP_OP_BMM && p.op != ALCOP_OP_CONV2D)
    return ALCOP_ERR_UNSUPPORTED;
  if (p.M <= 0 || p.N <= 0 || p.K <= 0 || p.batch <= 0 || p.batch > 65535) return ALCOP_ERR_SHAPE;
  if (p.N % 8 != 0 || p.K % 8 != 0) return ALCOP_ERR_SHAPE;
  if (p.transA && p.M % 8 != 0) return ALCOP_ERR_SHAPE;
  // convolution: transB selects the weight layout (0: RSCK = B stored K x N, 1: KRSC = N x K)
  if (p.op == ALCOP_OP_CONV2D &&
      (p.transA || p.conv_C <= 0 || p.conv_C % 8 != 0 || p.K % p.conv_C != 0))
    return ALCOP_ERR_SHAPE;
  return ALCOP_OK;
}

// Feasibility of a schedule for a problem (no pointers involved); sk = 1 looks among the
// split-K variants.
int check_sched(const alcop_problem& p, const alcop_sched& s, const KernelEntry** out, int sk = 0)
{
  int rc = check_problem(p);
  if (rc) return rc;
  if (s.stages < 1 || s.stages > 4 || s.reg_stages < 1 || s.reg_stages > 4) return ALCOP_ERR_SCHED;
  if (s.fuse_inner && (s.reg_stages < 2 || s.stages < 2)) return ALCOP_ERR_SCHED;
  // more than two register stages: only the fused pipeline, and its R-1 fragments in flight
  // must not reach beyond the next k-tile
  if (s.reg_stages > 2 && (!s.fuse_inner || (s.reg_stages - 1) * 16 > s.bk)) return ALCOP_ERR_SCHED;
  if (s.raster != 0 && s.raster != 1) return ALCOP_ERR_SCHED;
  if (s.l2_prefetch < 0 || s.l2_prefetch > 64 || (s.l2_prefetch > 0 && s.raster != 1))
    return ALCOP_ERR_SCHED;
  if (s.variant != 0 && s.variant != 2 &&
      !(s.variant == 1 && p.op == ALCOP_OP_CONV2D && !p.transB && p.conv_C == s.bk && sk == 0))
    return ALCOP_ERR_SCHED;
  // variant 2, the persistent producer / consumer kernels: two register stages (fused across
  // k-tiles and tiles, or restarted per k-tile) or four (three fragments in flight, fused, k-tiles
  // of 64 and more); no L2 touches, no split-K; convolutions with one tap per k-tile
  if (s.variant == 2 && ((s.reg_stages != 2 && !(s.reg_stages == 4 && s.fuse_inner)) || s.l2_prefetch != 0 || sk != 0 ||
                         s.stages < 2 || (p.op == ALCOP_OP_CONV2D && p.conv_C % s.bk != 0)))
    return ALCOP_ERR_SCHED;
  const KernelEntry* e = find_entry(p, s, sk);
  if (!e) return ALCOP_ERR_SCHED;
  if (e->lds_bytes > 160 * 1024) return ALCOP_ERR_SCHED;
  if (e->stages >= 2 && (e->stages - 2) * e->loads_per_stage > 63) return ALCOP_ERR_SCHED;
  // A partial last k-tile is zero-filled by the loader (K % 8 == 0 is checked with the problem).
  // Convolution: the channel count is a multiple of 8 (checked with the problem); which gather
  // a schedule gets follows from whether its k-tile divides the channel count.
  const long ntm = (p.M + s.bm - 1) / s.bm, ntn = (p.N + s.bn - 1) / s.bn;
  if (ntm * ntn > 0x7fffffffL) return ALCOP_ERR_SHAPE;
  if (out) *out = e;
  return ALCOP_OK;
}

// Depth of the HBM -> L2 level when it is on: look ahead 256 elements of k (a few L2 miss
// latencies of matrix work at any tile size).
int default_l2_prefetch(int bk) { return 256 / bk; }

// Kernels outside the default schedule space: offered to a caller who names them or asks the
// tuner for them, never picked by the model on its own.  These are the patch convolution (its
// feasibility depends on the call, not only on the problem description) and the kernels with a
// k-tile of 128 (two stages of a 128 x 128 tile fill the LDS: a trade the tuner should measure),
// and the persistent kernels with the consumers' deep register pipeline (no faster where measured).
bool opt_in(const KernelEntry& e) { return e.am == 3 || e.bk == 128 || (e.st && e.reg_stages == 4); }

// variants: 0 = the default kernels; 1 = also the opt-in kernels; 2 = only those.
std::vector<alcop_sched> space_of(const alcop_problem& p, int sk = 0, int variants = 0)
{
  std::vector<alcop_sched> v;
  for (const KernelEntry& e : registry())
    if (e.sk == sk && e.dt == (int)p.in && e.bl == (p.transB ? 1 : 0) &&
        e.al == (p.transA ? 1 : 0) &&
        (e.am == 3 ? (p.op == ALCOP_OP_CONV2D && p.conv_C == e.bk) : e.am == a_mode(p, e.bk, 0)) &&
        (variants == 1 || (variants == 2) == opt_in(e)))
    {
      // a kernel with the third (HBM -> L2) level is offered with that level on
      v.push_back(alcop_sched{e.bm, e.bn, e.bk, e.wm, e.wn, e.stages, e.reg_stages, e.fuse, 1,
                              e.pf ? default_l2_prefetch(e.bk) : 0, e.am == 3 ? 1 : (e.st ? 2 : 0)});
    }
  return v;
}

using CacheKey = std::tuple<int, int, int, int, int, int, int, int, int, int>;
std::mutex g_cache_mu;
std::map<CacheKey, alcop_sched> g_cache;   // problem -> chosen schedule (tuned or model top-1)

CacheKey key_of(const alcop_problem& p)
{
  return CacheKey{(int)p.op, p.batch, p.M, p.N, p.K, p.transB, (int)p.in, (int)p.out, p.conv_C,
                  p.transA};
}

int load_cache_file(const char* path);

// The static model's top-1 among the feasible default-variant schedules (variants that depend on
// more than the problem description, such as the patch convolution, are left to the tuner).
int model_pick(const alcop_problem& p, alcop_sched* out)
{
  const Device dev;
  double best = 0;
  bool have = false;
  for (const alcop_sched& s : space_of(p)) {
    if (check_sched(p, s, nullptr) != ALCOP_OK) continue;
    const double t = predict(p, s, 0, dev, nullptr);
    if (!have || t < best) {
      best = t;
      *out = s;
      have = true;
    }
  }
  return have ? ALCOP_OK : ALCOP_ERR_SCHED;
}

// What a NULL / zero schedule resolves to: the tuning cache, else the model's pick.
int auto_sched(const alcop_problem& p, alcop_sched* out)
{
  // a tuning cache named by the environment is merged in once, before the first lookup
  static std::once_flag env_once;
  std::call_once(env_once, [] {
    const char* path = std::getenv("ALCOP_TUNE_CACHE");
    if (path && *path) (void)load_cache_file(path);
  });
  {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    auto it = g_cache.find(key_of(p));
    if (it != g_cache.end()) {
      *out = it->second;
      return ALCOP_OK;
    }
  }
  const int rc = model_pick(p, out);
  if (rc) return rc;
  std::lock_guard<std::mutex> lk(g_cache_mu);
  g_cache[key_of(p)] = *out;
  return ALCOP_OK;
}

int check_call(const Call& c)
{
  if (!c.A || !c.B || !c.C) return ALCOP_ERR_NULL;
  int rc = check_problem(problem_of(c));
  if (rc) return rc;
  if (!aligned16(c.A) || !aligned16(c.B) || !aligned16(c.C)) return ALCOP_ERR_ALIGN;
  if (c.bias && !aligned16(c.bias)) return ALCOP_ERR_ALIGN;
  if (c.act != 0 && c.act != 1) return ALCOP_ERR_UNSUPPORTED;
  if (c.op == ALCOP_OP_CONV2D) {
    if (c.cR <= 0 || c.cS <= 0 || c.csh <= 0 || c.csw <= 0 || c.cph < 0 || c.cpw < 0 ||
        c.cP <= 0 || c.cQ <= 0 || c.cC % 8 != 0)
      return ALCOP_ERR_SHAPE;
    const double xbytes = 2.0 * c.cN * c.cH * c.cW * c.cC;
    if (xbytes >= 2147483648.0) return ALCOP_ERR_SIZE;
    return ALCOP_OK;
  }
  if ((c.lda | c.ldb | c.ldc) & 7) return ALCOP_ERR_ALIGN;
  if (c.batch > 1 && ((c.strideA | c.strideB | c.strideC) & 7)) return ALCOP_ERR_ALIGN;
  if (c.strideA < 0 || c.strideB < 0 || c.strideC < 0) return ALCOP_ERR_SHAPE;
  if (c.lda < (c.transA ? c.M : c.K) || c.ldb < (c.transB ? c.K : c.N) || c.ldc < c.N)
    return ALCOP_ERR_SHAPE;
  if (c.lda >= (1L << 30) || c.ldb >= (1L << 30) || c.ldc >= (1L << 30)) return ALCOP_ERR_SIZE;
  return ALCOP_OK;
}

int span_check(const Call& c, const alcop_sched& s)
{
  // The loaders form 32-bit byte offsets from a tile's origin.  For an operand whose rows run
  // along k (A stored K x M, B stored K x N) the rows of a partial last k-tile lie past the
  // descriptor and must stay below 2^31 as offsets, so that neither they nor the out-of-range
  // mark added to the loads of the ring's tail can wrap into the valid range: K is rounded up
  // to whole k-tiles there.
  const double rows = std::min(s.bm, c.M), cols = std::min(s.bn, c.N);
  const double kceil = (double)((c.K + s.bk - 1) / s.bk) * s.bk;
  const double a = c.op == ALCOP_OP_CONV2D ? 0.0   // x is checked as a whole with the call
                   : c.transA ? 2.0 * ((kceil - 1) * c.lda + rows) : 2.0 * ((rows - 1) * c.lda + c.K);
  const double b = c.transB ? 2.0 * ((cols - 1) * c.ldb + c.K) : 2.0 * ((kceil - 1) * c.ldb + cols);
  if (a >= 2147483648.0 || b >= 2147483648.0) return ALCOP_ERR_SIZE;
  return ALCOP_OK;
}

// Geometry of the patch variant of a convolution (schedule variant 1) for one call, or an error:
// stride 1; the patch (tile rows + halo, rounded up to whole block-wide loads) must fit the LDS.
struct Patch {
  int wp = 0, ntj = 0, loads = 0;
};
int patch_of(const Call& c, const alcop_sched& s, const KernelEntry* e, Patch* out)
{
  if (c.op != ALCOP_OP_CONV2D || c.csh != 1 || c.csw != 1 || c.cdh != 1 || c.cdw != 1)
    return ALCOP_ERR_SCHED;
  Patch pt;
  pt.wp = c.cW + 2 * c.cpw;                                    // row length of the padded image
  const long positions = (long)(c.cP - 1) * pt.wp + c.cQ;      // output positions per image
  pt.ntj = (int)((positions + s.bm - 1) / s.bm);
  const long rows = s.bm + (long)(c.cR - 1) * pt.wp + (c.cS - 1);
  const long slots = rows * (s.bk / 8);                        // 16-byte slots of the patch
  const long loads = (slots + e->threads - 1) / e->threads;
  if (e->patch_off + loads * e->threads * 16 > 160 * 1024) return ALCOP_ERR_SCHED;
  if ((long)pt.ntj * c.cN > 0x7fffffffL / std::max(1, (c.N + s.bn - 1) / s.bn)) return ALCOP_ERR_SHAPE;
  pt.loads = (int)loads;
  if (out) *out = pt;
  return ALCOP_OK;
}

// What a schedule needs from the call beyond the problem description.
int call_feasible(const Call& c, const alcop_sched& s, const KernelEntry* e)
{
  if (e->am == 3) return patch_of(c, s, e, nullptr);
  return ALCOP_OK;
}

// Slicing of the reduction axis for the split-K kernels: nz slices of len elements each (len is
// a multiple of the k-tile; the last slice may be shorter), fp32 partial tiles in ws.
struct Split {
  int nz = 1;
  int len = 0;
  void* ws = nullptr;
};

Split make_split(int K, int bk, int requested, void* ws)
{
  Split sp;
  const int nkt = (K + bk - 1) / bk;                            // k-tiles in all
  const int per = (nkt + requested - 1) / requested;            // k-tiles per slice
  sp.len = per * bk;
  sp.nz = (nkt + per - 1) / per;                                // no slice is empty
  sp.ws = ws;
  return sp;
}

// Compute units of the current device (256 on an MI355X; that number also when no device answers).
int compute_units()
{
  static std::once_flag once;
  static int n = 256;
  std::call_once(once, [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n = v;
  });
  return n;
}

int launch_call(const Call& c, const alcop_sched& s, const KernelEntry* e, hipStream_t st,
                const Split* split = nullptr)
{
  Params p;
  std::memset(&p, 0, sizeof(p));
  p.A = c.A;
  p.B = c.B;
  p.C = c.C;
  p.M = c.M;
  p.N = c.N;
  p.K = c.K;
  p.lda = (int)c.lda;
  p.ldb = (int)c.ldb;
  p.ldc = (int)c.ldc;
  p.strideA = c.strideA;
  p.strideB = c.strideB;
  p.strideC = c.strideC;
  p.out_dtype = (int)c.out;
  p.ntm = (c.M + s.bm - 1) / s.bm;
  p.ntn = (c.N + s.bn - 1) / s.bn;
  p.raster = s.raster;
  p.alpha = c.alpha;
  p.bias = (const float*)c.bias;
  p.act = c.act;
  p.group_m = std::min(8, p.ntm);
  // sharers of a panel among the blocks one XCD runs side by side (32 CUs, blocks per CU by LDS)
  const int per_cu = std::max(1, std::min(2, (160 * 1024) / e->lds_bytes));
  // The touch addresses of an M/N-contiguous operand walk whole k-tiles; with a partial last
  // k-tile some of them would lie past the operand's last row, so the level is switched off.
  p.pf_dist = (c.K % s.bk == 0) ? s.l2_prefetch : 0;
  p.pf_pb = std::max(1, p.group_m);
  p.pf_pa = std::max(1, std::min(p.ntn, 32 * per_cu / p.pf_pb));
  while (p.pf_pa > 1 && s.bm / p.pf_pa < 1) p.pf_pa--;
  if (c.op == ALCOP_OP_CONV2D) {
    p.cH = c.cH;
    p.cW = c.cW;
    p.cC = c.cC;
    p.cP = c.cP;
    p.cQ = c.cQ;
    p.cS = c.cS;
    p.csh = c.csh;
    p.csw = c.csw;
    p.cph = c.cph;
    p.cpw = c.cpw;
    p.cdh = c.cdh;
    p.cdw = c.cdw;
    p.a_span = (unsigned)(2L * c.cN * c.cH * c.cW * c.cC);
    if (e->am == 3) {
      Patch pt;
      if (patch_of(c, s, e, &pt) != ALCOP_OK) return ALCOP_ERR_SCHED;
      p.cR = c.cR;
      p.cWp = pt.wp;
      p.ntj = pt.ntj;
      p.patch_loads = pt.loads;
      p.ntm = pt.ntj * c.cN;                 // tiles of padded output positions, per image
      p.group_m = std::min(8, p.ntm);
    }
  }
  dim3 grid((unsigned)(p.ntm * p.ntn), (unsigned)c.batch, 1);
  if (e->st) {
    // persistent blocks: as many as stay resident (by LDS, at most two per compute unit), never
    // more than there are tiles; ALCOP_STREAM_BLOCKS overrides the count (a tuning and test knob)
    const long total = (long)p.ntm * p.ntn * c.batch;
    if (total > 0x7fffffffL) return ALCOP_ERR_SHAPE;
    long blocks = (long)compute_units() * std::max(1, std::min(2, (160 * 1024) / e->lds_bytes));
    if (const char* env = std::getenv("ALCOP_STREAM_BLOCKS")) {
      const long v = std::atol(env);
      if (v > 0) blocks = v;
    }
    p.sgrid = (int)std::min(total, blocks);
    p.sbatch = c.batch;
    grid = dim3((unsigned)p.sgrid, 1, 1);
  }
  if (split) {
    // the slices write plain fp32 tiles into the workspace; f(.) and the conversion to the
    // output type happen in the reduction step
    const long mn = (long)c.M * c.N;
    p.C = split->ws;
    p.ldc = c.N;
    p.strideC = mn;
    p.zstrideC = mn * c.batch;
    p.out_dtype = (int)ALCOP_F32;
    p.alpha = 1.0f;
    p.bias = nullptr;
    p.act = 0;
    p.pf_dist = 0;
    p.ksplit_len = split->len;
    grid.z = (unsigned)split->nz;
  }
  if (std::getenv("ALCOP_LOG"))
    std::fprintf(stderr,
                 "alcop: op %d M %d N %d K %d batch %d -> tile %dx%dx%d waves %dx%d S%d R%d F%d pf%d "
                 "variant %d%s grid (%u,%u,%u) threads %d lds %d\n",
                 (int)c.op, c.M, c.N, c.K, c.batch, s.bm, s.bn, s.bk, s.wm, s.wn, s.stages, s.reg_stages,
                 s.fuse_inner, s.l2_prefetch, s.variant, split ? " split-K" : "", grid.x, grid.y, grid.z,
                 e->threads, e->lds_bytes);
  hipError_t err = e->launch(p, grid, st);
  if (err != hipSuccess) return ALCOP_ERR_LAUNCH;
  if (split) {
    ReduceParams r;
    std::memset(&r, 0, sizeof(r));
    r.ws = (const float*)split->ws;
    r.C = c.C;
    r.M = c.M;
    r.N = c.N;
    r.ldc = (int)c.ldc;
    r.strideC = c.strideC;
    r.split = split->nz;
    r.zstride = (long)c.M * c.N * c.batch;
    r.out_dtype = (int)c.out;
    r.alpha = c.alpha;
    r.bias = (const float*)c.bias;
    r.act = c.act;
    const long threads = (long)c.M * (c.N / 8);
    dim3 rgrid((unsigned)((threads + REDUCE_THREADS - 1) / REDUCE_THREADS), (unsigned)c.batch, 1);
    err = launch_splitk_reduce(r, rgrid, st);
    if (err != hipSuccess) return ALCOP_ERR_LAUNCH;
  }
  return ALCOP_OK;
}

int run(const Call& c, const alcop_sched* sched, void* stream)
{
  int rc = check_call(c);
  if (rc) return rc;
  const alcop_problem prob = problem_of(c);
  alcop_sched s;
  const bool automatic = !sched || sched->bm == 0;
  if (automatic) {
    rc = auto_sched(prob, &s);
    if (rc) return rc;
  } else {
    s = *sched;
  }
  const KernelEntry* e = nullptr;
  rc = check_sched(prob, s, &e);
  if (rc) return rc;
  rc = span_check(c, s);
  if (rc) return rc;
  rc = call_feasible(c, s, e);
  if (rc && automatic && s.variant != 0) {
    // the cached schedule was tuned on a call with another geometry (the cache key is the
    // problem description): fall back to the model's pick for this call
    rc = model_pick(prob, &s);
    if (rc) return rc;
    rc = check_sched(prob, s, &e);
    if (rc) return rc;
    rc = span_check(c, s);
    if (rc) return rc;
    rc = call_feasible(c, s, e);
  }
  if (rc) return rc;
  return launch_call(c, s, e, (hipStream_t)stream);
}

// Predicted time of a split-K schedule: the main loop as a problem with batch x nz blocks over
// a reduction axis of one slice and fp32 output, plus the reduction pass (one launch latency and
// its traffic at DRAM rate).  Same model, applied to the transformed problem.
double predict_splitk(const alcop_problem& p, const alcop_sched& s, int requested, const Device& dev)
{
  const Split sp = make_split(p.K, s.bk, requested, nullptr);
  alcop_problem q = p;
  q.batch = p.batch * sp.nz;
  q.K = sp.len;
  q.out = ALCOP_F32;
  double t = predict(q, s, 0, dev, nullptr);
  if (sp.nz > 1) {
    const double out_b = p.out == ALCOP_F32 ? 4.0 : 2.0;
    const double bytes = (double)p.batch * p.M * p.N * (4.0 * sp.nz + out_b);
    t += dev.lat_dram + dev.lat_dram_write + bytes / dev.bw_dram;
  }
  return t;
}

const int kSplitChoices[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32};

// Model's pick of (schedule, split) among the split-K variants; split = 0 searches it too.
int auto_splitk(const alcop_problem& p, int split, alcop_sched* out, int* split_out)
{
  const Device dev;
  double best = 0;
  bool have = false;
  for (const alcop_sched& s : space_of(p, 1)) {
    if (check_sched(p, s, nullptr, 1) != ALCOP_OK) continue;
    auto consider = [&](int n) {
      const double t = predict_splitk(p, s, n, dev);
      if (!have || t < best) {
        best = t;
        *out = s;
        *split_out = n;
        have = true;
      }
    };
    if (split > 0) {
      consider(split);
      continue;
    }
    for (int cand : kSplitChoices)
      if (cand <= (p.K + s.bk - 1) / s.bk) consider(cand);
  }
  return have ? ALCOP_OK : ALCOP_ERR_SCHED;
}

static_assert(kSplitkStaticBytes == ALCOP_SPLITK_STATIC_BYTES, "scratch size: header and device array");

// ws == nullptr with own_scratch: the partial tiles go to the library's own device array.
int run_splitk(const Call& c, const alcop_sched* sched, int split, void* ws, size_t ws_bytes,
               void* stream, bool own_scratch = false)
{
  int rc = check_call(c);
  if (rc) return rc;
  if (split < 0 || split > 64) return ALCOP_ERR_SHAPE;
  if (own_scratch) {
    ws_bytes = ALCOP_SPLITK_STATIC_BYTES;
  } else {
    if (!ws) return ALCOP_ERR_NULL;
    if (!aligned16(ws)) return ALCOP_ERR_ALIGN;
  }
  const alcop_problem prob = problem_of(c);
  alcop_sched s;
  if (!sched || sched->bm == 0) {
    rc = auto_splitk(prob, split, &s, &split);
    if (rc) return rc;
  } else {
    s = *sched;
    if (split == 0) {
      alcop_sched ignored;
      rc = auto_splitk(prob, 0, &ignored, &split);
      if (rc) return rc;
    }
  }
  const KernelEntry* e = nullptr;
  rc = check_sched(prob, s, &e, 1);
  if (rc) return rc;
  if (s.l2_prefetch != 0) return ALCOP_ERR_SCHED;
  rc = span_check(c, s);
  if (rc) return rc;
  Split sp = make_split(c.K, s.bk, split, ws);
  const double need = 4.0 * sp.nz * c.batch * c.M * c.N;
  if (need > (double)ws_bytes) return ALCOP_ERR_SIZE;
  if (own_scratch) {
    // sizes are settled; only now touch the device (the first call per device looks the array up)
    void* mine = nullptr;
    size_t have = 0;
    if (splitk_scratch(&mine, &have) != hipSuccess || need > (double)have) return ALCOP_ERR_LAUNCH;
    sp.ws = mine;
  }
  return launch_call(c, s, e, (hipStream_t)stream, &sp);
}

Call gemm_call(alcop_op op, const void* A, const void* B, void* C, int batch, int M, int N, int K,
               long lda, long ldb, long ldc, long sA, long sB, long sC, int transA, int transB,
               alcop_dtype in, alcop_dtype out)
{
  Call c;
  std::memset(&c, 0, sizeof(c));
  c.op = op;
  c.A = A;
  c.B = B;
  c.C = C;
  c.batch = batch;
  c.M = M;
  c.N = N;
  c.K = K;
  c.lda = lda;
  c.ldb = ldb;
  c.ldc = ldc;
  c.strideA = sA;
  c.strideB = sB;
  c.strideC = sC;
  c.transA = transA ? 1 : 0;
  c.transB = transB ? 1 : 0;
  c.in = in;
  c.out = out;
  c.alpha = 1.0f;
  return c;
}

// Order of the trials of a fixed-ranking tuning run: by predicted latency, but among the first
// top_k at most max(2, top_k / 4) schedules of one (tile, wave tile, variant) family.  The
// pipelining variants of one tile are predicted within a few percent of each other; without the
// cap the near-ties of one tile fill the whole budget and a mispredicted tile costs the run.
template <class Cand>
void spread_over_tiles(std::vector<Cand>& ranked, int top_k)
{
  if (top_k <= 0 || (int)ranked.size() <= top_k) return;
  const int cap = std::max(2, top_k / 4);
  std::map<std::tuple<int, int, int, int, int, int>, int> taken;
  std::vector<Cand> head, tail;
  for (const Cand& cd : ranked) {
    const alcop_sched& s = cd.s;
    int& n = taken[std::make_tuple(s.bm, s.bn, s.bk, s.wm, s.wn, s.variant)];
    if ((int)head.size() < top_k && n < cap) {
      n++;
      head.push_back(cd);
    } else {
      tail.push_back(cd);
    }
  }
  // Insurance against the case the paper reports in Sec. 6.2 (pipelining slows some operators
  // down): with a budget of 8 or more, the budget's last trials go to the unpipelined (one-stage)
  // schedule of the two best-ranked tile-at-a-time tile families, unless it holds one already.
  if (top_k >= 8) {
    std::vector<std::tuple<int, int, int, int, int, int>> fams;
    for (const Cand& cd : head) {
      const alcop_sched& s = cd.s;
      if (s.variant == 2) continue;   // persistent kernels have no one-stage form
      const auto f = std::make_tuple(s.bm, s.bn, s.bk, s.wm, s.wn, s.variant);
      if (std::find(fams.begin(), fams.end(), f) == fams.end()) fams.push_back(f);
      if (fams.size() == 2) break;
    }
    std::vector<Cand> ins;
    for (const auto& f : fams) {
      auto of_family = [&](const Cand& cd) {
        const alcop_sched& s = cd.s;
        return std::make_tuple(s.bm, s.bn, s.bk, s.wm, s.wn, s.variant) == f && s.stages == 1;
      };
      if (std::any_of(head.begin(), head.end(), of_family)) continue;
      auto it = std::find_if(tail.begin(), tail.end(), of_family);
      if (it == tail.end()) continue;
      // the model does not tell the one-stage schedules of a tile apart: take the one that still
      // prefetches its fragments (R = 2), which costs nothing and is never slower
      auto r2 = std::find_if(tail.begin(), tail.end(),
                             [&](const Cand& cd) { return of_family(cd) && cd.s.reg_stages == 2; });
      if (r2 != tail.end()) it = r2;
      ins.push_back(*it);
      tail.erase(it);
    }
    if (ins.size() < head.size()) {
      tail.insert(tail.begin(), head.end() - (long)ins.size(), head.end());
      head.resize(head.size() - ins.size());
      head.insert(head.end(), ins.begin(), ins.end());
    }
  }
  head.insert(head.end(), tail.begin(), tail.end());
  ranked.swap(head);
}

int conv_call(Call* c, const void* x, const void* w, void* y, int N, int H, int W, int Cc, int K,
              int R, int S, int sh, int sw, int ph, int pw, alcop_dtype in, alcop_dtype out,
              int krsc = 0, int dh = 1, int dw = 1)
{
  std::memset(c, 0, sizeof(*c));
  if (N <= 0 || H <= 0 || W <= 0 || Cc <= 0 || K <= 0 || R <= 0 || S <= 0 || sh <= 0 || sw <= 0 ||
      ph < 0 || pw < 0 || dh <= 0 || dw <= 0)
    return ALCOP_ERR_SHAPE;
  // extent of the dilated filter: dil * (R - 1) + 1
  const long eh = (long)dh * (R - 1) + 1, ew = (long)dw * (S - 1) + 1;
  if (H + 2L * ph < eh || W + 2L * pw < ew) return ALCOP_ERR_SHAPE;
  const long P = (H + 2L * ph - eh) / sh + 1, Q = (W + 2L * pw - ew) / sw + 1;
  const long Mg = (long)N * P * Q, Kg = (long)R * S * Cc;
  if (Mg > 0x7fffffffL || Kg > 0x7fffffffL) return ALCOP_ERR_SHAPE;
  c->op = ALCOP_OP_CONV2D;
  c->A = x;
  c->B = w;
  c->C = y;
  c->batch = 1;
  c->M = (int)Mg;
  c->N = K;
  c->K = (int)Kg;
  c->lda = Kg;
  c->ldb = krsc ? Kg : K;
  c->ldc = K;
  c->transB = krsc ? 1 : 0;
  c->in = in;
  c->out = out;
  c->cN = N;
  c->cH = H;
  c->cW = W;
  c->cC = Cc;
  c->cK = K;
  c->cR = R;
  c->cS = S;
  c->csh = sh;
  c->csw = sw;
  c->cph = ph;
  c->cpw = pw;
  c->cP = (int)P;
  c->cQ = (int)Q;
  c->cdh = dh;
  c->cdw = dw;
  c->alpha = 1.0f;
  return ALCOP_OK;
}

// Builds the Call of a model/tuner-style request (problem + operand pointers).
int call_of_problem(const alcop_problem* prob, const void* A, const void* B, void* C, long lda,
                    long ldb, long ldc, long sA, long sB, long sC, const int* conv, Call* out)
{
  if (!prob) return ALCOP_ERR_NULL;
  if (prob->op == ALCOP_OP_CONV2D) {
    if (!conv) return ALCOP_ERR_NULL;
    int rc = conv_call(out, A, B, C, conv[0], conv[1], conv[2], conv[3], conv[4], conv[5], conv[6],
                       conv[7], conv[8], conv[9], conv[10], prob->in, prob->out, prob->transB);
    if (rc) return rc;
    if (out->M != prob->M || out->N != prob->N || out->K != prob->K) return ALCOP_ERR_SHAPE;
    return ALCOP_OK;
  }
  *out = gemm_call(prob->op, A, B, C, prob->batch, prob->M, prob->N, prob->K, lda, ldb, ldc, sA,
                   sB, sC, prob->transA, prob->transB, prob->in, prob->out);
  return ALCOP_OK;
}

// Mean microseconds per launch over `iters` back-to-back launches (HIP events on `st`).
int time_sched(const Call& c, const alcop_sched& s, const KernelEntry* e, int warmup, int iters,
               hipStream_t st, double* us, const Split* split = nullptr)
{
  for (int i = 0; i < warmup; i++) {
    int rc = launch_call(c, s, e, st, split);
    if (rc) return rc;
  }
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return ALCOP_ERR_LAUNCH;
  if (hipEventCreate(&e1) != hipSuccess) {
    (void)hipEventDestroy(e0);
    return ALCOP_ERR_LAUNCH;
  }
  int rc = ALCOP_OK;
  (void)hipEventRecord(e0, st);
  for (int i = 0; i < iters && rc == ALCOP_OK; i++) rc = launch_call(c, s, e, st, split);
  (void)hipEventRecord(e1, st);
  if (hipEventSynchronize(e1) != hipSuccess) rc = ALCOP_ERR_LAUNCH;
  float ms = 0.f;
  if (rc == ALCOP_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = ALCOP_ERR_LAUNCH;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc == ALCOP_OK) *us = (double)ms * 1000.0 / iters;
  return rc;
}


// ---- operands the loops cannot take as they are: padded images in a workspace (alcop_pack.hip.h)
inline long r8(long x) { return (x + 7) & ~7L; }
inline size_t r256(double bytes) { return ((size_t)bytes + 255) & ~(size_t)255; }
inline int out_size(alcop_dtype out) { return out == ALCOP_F32 ? 4 : 2; }

// Sections of the workspace: padded A, padded B, padded C, padded bias.  Returns the total, or 0
// if a section would reach 2 GiB (the kernels' 32-bit offsets) or the total overflows.
size_t unaligned_layout(double a_elems, double b_elems, double c_elems, long n8, alcop_dtype out,
                        size_t off[4])
{
  const double a = 2.0 * a_elems, b = 2.0 * b_elems, c = (double)out_size(out) * c_elems;
  if (a >= 2147483648.0 || b >= 2147483648.0 || c >= 4294967296.0) return 0;
  off[0] = 0;
  off[1] = off[0] + r256(a);
  off[2] = off[1] + r256(b);
  off[3] = off[2] + r256(c);
  return off[3] + r256(4.0 * (double)n8);
}

PackParams pack2d(const void* src, void* dst, int rows, int cols, long s_batch, long s_row, int rows_d,
                  int cols_d, long d_batch, long d_row, int esize)
{
  PackParams p;
  p.src = src;
  p.dst = dst;
  p.rows = rows;
  p.cols = cols;
  p.s_batch = s_batch;
  p.s_row = s_row;
  p.rows_d = rows_d;
  p.cols_d = cols_d;
  p.d_batch = d_batch;
  p.d_row = d_row;
  p.esize = esize;
  return p;
}

bool elem_aligned(const void* p, int esize) { return (reinterpret_cast<uintptr_t>(p) & (uintptr_t)(esize - 1)) == 0; }

// Padded bias (N8 floats, zero tail) if the epilogue has one; fills the inner call's epilogue.
int pack_epilogue(const alcop_epilogue* ep, int N, char* ws_bias, Call* inner, hipStream_t st)
{
  if (!ep) return ALCOP_OK;
  inner->alpha = ep->alpha;
  inner->act = ep->act;
  if (ep->act != 0 && ep->act != 1) return ALCOP_ERR_UNSUPPORTED;
  if (ep->bias) {
    if (!elem_aligned(ep->bias, 4)) return ALCOP_ERR_ALIGN;
    const int n8 = (int)r8(N);
    if (launch_pack(pack2d(ep->bias, ws_bias, 1, N, 0, 0, 1, n8, 0, n8, 4), 1, st) != hipSuccess)
      return ALCOP_ERR_LAUNCH;
    inner->bias = ws_bias;
  }
  return ALCOP_OK;
}

}  // namespace
}  // namespace alcop

using namespace alcop;

extern "C" {

int alcop_gemm(const void* A, const void* B, void* C, int M, int N, int K, long lda, long ldb,
               long ldc, int transA, int transB, alcop_dtype in, alcop_dtype out,
               const alcop_sched* sched, void* hip_stream)
{
  Call c = gemm_call(ALCOP_OP_GEMM, A, B, C, 1, M, N, K, lda, ldb, ldc, 0, 0, 0, transA, transB, in, out);
  return run(c, sched, hip_stream);
}

int alcop_bmm(const void* A, const void* B, void* C, int batch, int M, int N, int K, long lda,
              long ldb, long ldc, long strideA, long strideB, long strideC, int transA, int transB,
              alcop_dtype in, alcop_dtype out, const alcop_sched* sched, void* hip_stream)
{
  Call c = gemm_call(ALCOP_OP_BMM, A, B, C, batch, M, N, K, lda, ldb, ldc, strideA, strideB,
                     strideC, transA, transB, in, out);
  return run(c, sched, hip_stream);
}

int alcop_gemm_fused(const void* A, const void* B, void* C, int M, int N, int K, long lda, long ldb,
                     long ldc, int transA, int transB, alcop_dtype in, alcop_dtype out,
                     const alcop_epilogue* ep, const alcop_sched* sched, void* hip_stream)
{
  Call c = gemm_call(ALCOP_OP_GEMM, A, B, C, 1, M, N, K, lda, ldb, ldc, 0, 0, 0, transA, transB, in, out);
  if (ep) {
    c.alpha = ep->alpha;
    c.bias = ep->bias;
    c.act = ep->act;
  }
  return run(c, sched, hip_stream);
}

int alcop_bmm_fused(const void* A, const void* B, void* C, int batch, int M, int N, int K, long lda,
                    long ldb, long ldc, long strideA, long strideB, long strideC, int transA,
                    int transB, alcop_dtype in, alcop_dtype out, const alcop_epilogue* ep,
                    const alcop_sched* sched, void* hip_stream)
{
  Call c = gemm_call(ALCOP_OP_BMM, A, B, C, batch, M, N, K, lda, ldb, ldc, strideA, strideB,
                     strideC, transA, transB, in, out);
  if (ep) {
    c.alpha = ep->alpha;
    c.bias = ep->bias;
    c.act = ep->act;
  }
  return run(c, sched, hip_stream);
}

int alcop_conv2d_igemm(const void* x, const void* w, void* y, int N, int H, int W, int C, int K,
                       int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                       alcop_dtype in, alcop_dtype out, const alcop_sched* sched, void* hip_stream)
{
  Call c;
  int rc = conv_call(&c, x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, in, out);
  if (rc) return rc;
  return run(c, sched, hip_stream);
}

int alcop_conv2d_igemm_dilated(const void* x, const void* w, void* y, int N, int H, int W, int C,
                               int K, int R, int S, int stride_h, int stride_w, int pad_h,
                               int pad_w, int dil_h, int dil_w, int krsc, alcop_dtype in,
                               alcop_dtype out, const alcop_epilogue* ep, const alcop_sched* sched,
                               void* hip_stream)
{
  Call c;
  int rc = conv_call(&c, x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, in, out,
                     krsc ? 1 : 0, dil_h, dil_w);
  if (rc) return rc;
  if (ep) {
    c.alpha = ep->alpha;
    c.bias = ep->bias;
    c.act = ep->act;
  }
  return run(c, sched, hip_stream);
}

size_t alcop_splitk_workspace_bytes(int batch, int M, int N, int split)
{
  if (batch <= 0 || M <= 0 || N <= 0 || split <= 0) return 0;
  return (size_t)4 * (size_t)split * (size_t)batch * (size_t)M * (size_t)N;
}

int alcop_gemm_splitk(const void* A, const void* B, void* C, int batch, int M, int N, int K,
                      long lda, long ldb, long ldc, long strideA, long strideB, long strideC,
                      int transA, int transB, alcop_dtype in, alcop_dtype out,
                      const alcop_epilogue* ep, const alcop_sched* sched, int split,
                      void* workspace, size_t workspace_bytes, void* hip_stream)
{
  Call c = gemm_call(batch > 1 ? ALCOP_OP_BMM : ALCOP_OP_GEMM, A, B, C, batch, M, N, K, lda, ldb, ldc,
                     strideA, strideB, strideC, transA, transB, in, out);
  if (ep) {
    c.alpha = ep->alpha;
    c.bias = ep->bias;
    c.act = ep->act;
  }
  return run_splitk(c, sched, split, workspace, workspace_bytes, hip_stream);
}

int alcop_gemm_splitk_static(const void* A, const void* B, void* C, int batch, int M, int N, int K,
                             long lda, long ldb, long ldc, long strideA, long strideB,
                             long strideC, int transA, int transB, alcop_dtype in, alcop_dtype out,
                             const alcop_epilogue* ep, const alcop_sched* sched, int split,
                             void* hip_stream)
{
  Call c = gemm_call(batch > 1 ? ALCOP_OP_BMM : ALCOP_OP_GEMM, A, B, C, batch, M, N, K, lda, ldb, ldc,
                     strideA, strideB, strideC, transA, transB, in, out);
  if (ep) {
    c.alpha = ep->alpha;
    c.bias = ep->bias;
    c.act = ep->act;
  }
  return run_splitk(c, sched, split, nullptr, 0, hip_stream, true);
}

int alcop_conv2d_igemm_splitk(const void* x, const void* w, void* y, int N, int H, int W, int C,
                              int K, int R, int S, int stride_h, int stride_w, int pad_h,
                              int pad_w, alcop_dtype in, alcop_dtype out, const alcop_sched* sched,
                              int split, void* workspace, size_t workspace_bytes, void* hip_stream)
{
  Call c;
  int rc = conv_call(&c, x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, in, out);
  if (rc) return rc;
  return run_splitk(c, sched, split, workspace, workspace_bytes, hip_stream);
}

int alcop_tune_splitk(const alcop_problem* prob, const void* A, const void* B, void* C, long lda,
                      long ldb, long ldc, long strideA, long strideB, long strideC, const int* conv,
                      void* workspace, size_t workspace_bytes, int top_k, int iters,
                      alcop_sched* best, int* best_split, double* best_us, int* trials_run,
                      int* space_size, alcop_sched* log_sched, int* log_split, double* log_pred_us,
                      double* log_meas_us, int log_cap, void* hip_stream)
{
  if (!best || !best_split || !best_us) return ALCOP_ERR_NULL;
  if (!workspace) return ALCOP_ERR_NULL;
  if (!aligned16(workspace)) return ALCOP_ERR_ALIGN;
  if (top_k < 0 || iters <= 0) return ALCOP_ERR_SHAPE;
  Call c;
  int rc = call_of_problem(prob, A, B, C, lda, ldb, ldc, strideA, strideB, strideC, conv, &c);
  if (rc) return rc;
  rc = check_call(c);
  if (rc) return rc;
  const alcop_problem p = problem_of(c);
  struct Cand {
    alcop_sched s;
    const KernelEntry* e;
    Split sp;
    double pred;
  };
  std::vector<Cand> cands;
  const Device dev;
  for (const alcop_sched& s : space_of(p, 1)) {
    const KernelEntry* e = nullptr;
    if (check_sched(p, s, &e, 1) != ALCOP_OK || span_check(c, s) != ALCOP_OK) continue;
    int last_nz = 0;
    for (int k : kSplitChoices) {
      const Split sp = make_split(c.K, s.bk, k, workspace);
      if (sp.nz == last_nz) continue;                       // same slicing as a smaller request
      last_nz = sp.nz;
      if (4.0 * sp.nz * c.batch * c.M * c.N > (double)workspace_bytes) continue;   // pruned
      cands.push_back(Cand{s, e, sp, predict_splitk(p, s, k, dev)});
    }
  }
  if (space_size) *space_size = (int)cands.size();
  if (cands.empty()) return ALCOP_ERR_SCHED;
  std::stable_sort(cands.begin(), cands.end(),
                   [](const Cand& a, const Cand& b) { return a.pred < b.pred; });
  const int n = top_k == 0 ? (int)cands.size() : std::min(top_k, (int)cands.size());
  bool have = false;
  for (int t = 0; t < n; t++) {
    double us = 0;
    rc = time_sched(c, cands[t].s, cands[t].e, 3, iters, (hipStream_t)hip_stream, &us, &cands[t].sp);
    if (rc) return rc;
    if (t < log_cap) {
      if (log_sched) log_sched[t] = cands[t].s;
      if (log_split) log_split[t] = cands[t].sp.nz;
      if (log_pred_us) log_pred_us[t] = cands[t].pred;
      if (log_meas_us) log_meas_us[t] = us;
    }
    if (!have || us < *best_us) {
      *best_us = us;
      *best = cands[t].s;
      *best_split = cands[t].sp.nz;
      have = true;
    }
  }
  if (trials_run) *trials_run = n;
  return ALCOP_OK;
}

int alcop_splitk_space(const alcop_problem* prob, alcop_sched* out, int cap)
{
  if (!prob) return ALCOP_ERR_NULL;
  const int rc = check_problem(*prob);
  if (rc) return rc;
  const std::vector<alcop_sched> v = space_of(*prob, 1);
  if (out)
    for (int i = 0; i < (int)v.size() && i < cap; i++) out[i] = v[i];
  return (int)v.size();
}

int alcop_splitk_auto(const alcop_problem* prob, int split, alcop_sched* sched_out, int* split_out,
                      double* predicted_us)
{
  if (!prob || !sched_out || !split_out) return ALCOP_ERR_NULL;
  int rc = check_problem(*prob);
  if (rc) return rc;
  if (split < 0 || split > 64) return ALCOP_ERR_SHAPE;
  rc = auto_splitk(*prob, split, sched_out, split_out);
  if (rc) return rc;
  if (predicted_us) *predicted_us = predict_splitk(*prob, *sched_out, *split_out, Device());
  return ALCOP_OK;
}

int alcop_conv2d_igemm_krsc(const void* x, const void* w, void* y, int N, int H, int W, int C,
                            int K, int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                            alcop_dtype in, alcop_dtype out, const alcop_sched* sched,
                            void* hip_stream)
{
  Call c;
  int rc = conv_call(&c, x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, in, out, 1);
  if (rc) return rc;
  return run(c, sched, hip_stream);
}

int alcop_conv2d_igemm_fused(const void* x, const void* w, void* y, int N, int H, int W, int C,
                             int K, int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                             alcop_dtype in, alcop_dtype out, const alcop_epilogue* ep, int krsc,
                             const alcop_sched* sched, void* hip_stream)
{
  Call c;
  int rc = conv_call(&c, x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, in, out,
                     krsc ? 1 : 0);
  if (rc) return rc;
  if (ep) {
    c.alpha = ep->alpha;
    c.bias = ep->bias;
    c.act = ep->act;
  }
  return run(c, sched, hip_stream);
}

int alcop_init(void)
{
  // everything a first call would do besides launching: the LDS opt-in of every kernel, the
  // address of the allocation-free entry point's device array, the compute-unit count
  for (const KernelEntry& e : registry())
    if (e.prepare && e.prepare() != hipSuccess) return ALCOP_ERR_LAUNCH;
  void* scratch = nullptr;
  size_t bytes = 0;
  if (splitk_scratch(&scratch, &bytes) != hipSuccess) return ALCOP_ERR_LAUNCH;
  (void)compute_units();
  return ALCOP_OK;
}

size_t alcop_unaligned_workspace_bytes(int batch, int M, int N, int K, alcop_dtype out)
{
  if (batch <= 0 || M <= 0 || N <= 0 || K <= 0) return 0;
  if (out != ALCOP_F16 && out != ALCOP_BF16 && out != ALCOP_F32) return 0;
  const double b = batch, m8 = (double)r8(M), n8 = (double)r8(N), k8 = (double)r8(K);
  size_t off[4];
  return unaligned_layout(b * m8 * k8, b * k8 * n8, b * m8 * n8, r8(N), out, off);
}

int alcop_bmm_unaligned(const void* A, const void* B, void* C, int batch, int M, int N, int K, long lda,
                        long ldb, long ldc, long strideA, long strideB, long strideC, int transA,
                        int transB, alcop_dtype in, alcop_dtype out, const alcop_epilogue* ep,
                        const alcop_sched* sched, void* workspace, size_t workspace_bytes,
                        void* hip_stream)
{
  if (!A || !B || !C || !workspace) return ALCOP_ERR_NULL;
  if (in != ALCOP_F16 && in != ALCOP_BF16) return ALCOP_ERR_DTYPE;
  if (out != ALCOP_F16 && out != ALCOP_BF16 && out != ALCOP_F32) return ALCOP_ERR_DTYPE;
  if (batch <= 0 || batch > 65535 || M <= 0 || N <= 0 || K <= 0) return ALCOP_ERR_SHAPE;
  transA = transA ? 1 : 0;
  transB = transB ? 1 : 0;
  if (lda < (transA ? M : K) || ldb < (transB ? K : N) || ldc < N) return ALCOP_ERR_SHAPE;
  if (strideA < 0 || strideB < 0 || strideC < 0) return ALCOP_ERR_SHAPE;
  const int osz = out_size(out);
  if (!elem_aligned(A, 2) || !elem_aligned(B, 2) || !elem_aligned(C, osz) || !aligned16(workspace))
    return ALCOP_ERR_ALIGN;
  const int m8 = (int)r8(M), n8 = (int)r8(N), k8 = (int)r8(K);
  size_t off[4];
  const size_t need = unaligned_layout((double)batch * m8 * k8, (double)batch * k8 * n8,
                                       (double)batch * m8 * n8, n8, out, off);
  if (need == 0 || workspace_bytes < need) return ALCOP_ERR_SIZE;
  char* ws = (char*)workspace;
  hipStream_t st = (hipStream_t)hip_stream;
  // padded operands, each batch entry a dense matrix
  const int a_rows = transA ? K : M, a_cols = transA ? M : K, a_rd = transA ? k8 : m8, a_cd = transA ? m8 : k8;
  const int b_rows = transB ? N : K, b_cols = transB ? K : N, b_rd = transB ? n8 : k8, b_cd = transB ? k8 : n8;
  Call c = gemm_call(batch > 1 ? ALCOP_OP_BMM : ALCOP_OP_GEMM, ws + off[0], ws + off[1], ws + off[2],
                     batch, m8, n8, k8, a_cd, b_cd, n8, (long)m8 * k8, (long)k8 * n8, (long)m8 * n8,
                     transA, transB, in, out);
  int rc = pack_epilogue(ep, N, ws + off[3], &c, st);
  if (rc) return rc;
  if (launch_pack(pack2d(A, ws + off[0], a_rows, a_cols, strideA, lda, a_rd, a_cd, (long)m8 * k8, a_cd, 2),
                  batch, st) != hipSuccess ||
      launch_pack(pack2d(B, ws + off[1], b_rows, b_cols, strideB, ldb, b_rd, b_cd, (long)k8 * n8, b_cd, 2),
                  batch, st) != hipSuccess)
    return ALCOP_ERR_LAUNCH;
  rc = run(c, sched, hip_stream);
  if (rc) return rc;
  if (launch_unpack(pack2d(ws + off[2], C, M, N, (long)m8 * n8, n8, m8, n8, strideC, ldc, osz), batch, st) !=
      hipSuccess)
    return ALCOP_ERR_LAUNCH;
  return ALCOP_OK;
}

// Output extent of the convolution, or false if the arguments do not describe one.
static bool conv_extent(int N, int H, int W, int C, int K, int R, int S, int sh, int sw, int ph, int pw,
                        int dh, int dw, long* P, long* Q)
{
  if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || K <= 0 || R <= 0 || S <= 0 || sh <= 0 || sw <= 0 ||
      ph < 0 || pw < 0 || dh <= 0 || dw <= 0)
    return false;
  const long eh = (long)dh * (R - 1) + 1, ew = (long)dw * (S - 1) + 1;
  if (H + 2L * ph < eh || W + 2L * pw < ew) return false;
  *P = (H + 2L * ph - eh) / sh + 1;
  *Q = (W + 2L * pw - ew) / sw + 1;
  return true;
}

size_t alcop_conv2d_unaligned_workspace_bytes(int N, int H, int W, int C, int K, int R, int S,
                                              int stride_h, int stride_w, int pad_h, int pad_w,
                                              int dil_h, int dil_w, alcop_dtype out)
{
  long P, Q;
  if (!conv_extent(N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, &P, &Q)) return 0;
  if (out != ALCOP_F16 && out != ALCOP_BF16 && out != ALCOP_F32) return 0;
  const double c8 = (double)r8(C), k8 = (double)r8(K);
  size_t off[4];
  return unaligned_layout((double)N * H * W * c8, (double)R * S * c8 * k8, (double)N * P * Q * k8, r8(K),
                          out, off);
}

int alcop_conv2d_igemm_unaligned(const void* x, const void* w, void* y, int N, int H, int W, int C,
                                 int K, int R, int S, int stride_h, int stride_w, int pad_h,
                                 int pad_w, int dil_h, int dil_w, alcop_dtype in, alcop_dtype out,
                                 const alcop_epilogue* ep, const alcop_sched* sched, void* workspace,
                                 size_t workspace_bytes, void* hip_stream)
{
  if (!x || !w || !y || !workspace) return ALCOP_ERR_NULL;
  if (in != ALCOP_F16 && in != ALCOP_BF16) return ALCOP_ERR_DTYPE;
  if (out != ALCOP_F16 && out != ALCOP_BF16 && out != ALCOP_F32) return ALCOP_ERR_DTYPE;
  long P, Q;
  if (!conv_extent(N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, &P, &Q))
    return ALCOP_ERR_SHAPE;
  const int osz = out_size(out);
  if (!elem_aligned(x, 2) || !elem_aligned(w, 2) || !elem_aligned(y, osz) || !aligned16(workspace))
    return ALCOP_ERR_ALIGN;
  const int c8 = (int)r8(C), k8 = (int)r8(K);
  const long pixels = (long)N * H * W, outputs = (long)N * P * Q;
  if (pixels > 0x7fffffffL || outputs > 0x7fffffffL) return ALCOP_ERR_SHAPE;
  size_t off[4];
  const size_t need = unaligned_layout((double)pixels * c8, (double)R * S * c8 * k8, (double)outputs * k8,
                                       k8, out, off);
  if (need == 0 || workspace_bytes < need) return ALCOP_ERR_SIZE;
  char* ws = (char*)workspace;
  hipStream_t st = (hipStream_t)hip_stream;
  Call c;
  int rc = conv_call(&c, ws + off[0], ws + off[1], ws + off[2], N, H, W, c8, k8, R, S, stride_h, stride_w,
                     pad_h, pad_w, in, out, 0, dil_h, dil_w);
  if (rc) return rc;
  rc = pack_epilogue(ep, K, ws + off[3], &c, st);
  if (rc) return rc;
  // x: pixels x C -> pixels x C8; w: (R*S) matrices of C x K -> C8 x K8
  if (launch_pack(pack2d(x, ws + off[0], (int)pixels, C, 0, C, (int)pixels, c8, 0, c8, 2), 1, st) != hipSuccess ||
      launch_pack(pack2d(w, ws + off[1], C, K, (long)C * K, K, c8, k8, (long)c8 * k8, k8, 2), R * S, st) !=
          hipSuccess)
    return ALCOP_ERR_LAUNCH;
  rc = run(c, sched, hip_stream);
  if (rc) return rc;
  if (launch_unpack(pack2d(ws + off[2], y, (int)outputs, K, 0, k8, (int)outputs, k8, 0, K, osz), 1, st) !=
      hipSuccess)
    return ALCOP_ERR_LAUNCH;
  return ALCOP_OK;
}

int alcop_sched_supported(const alcop_problem* prob, const alcop_sched* sched)
{
  if (!prob || !sched) return ALCOP_ERR_NULL;
  return check_sched(*prob, *sched, nullptr);
}

int alcop_sched_space(const alcop_problem* prob, alcop_sched* out, int cap)
{
  if (!prob) return ALCOP_ERR_NULL;
  const int rc = check_problem(*prob);
  if (rc) return rc;
  const std::vector<alcop_sched> v = space_of(*prob);
  if (out)
    for (int i = 0; i < (int)v.size() && i < cap; i++) out[i] = v[i];
  return (int)v.size();
}

int alcop_model_predict(const alcop_problem* prob, const alcop_sched* sched, int model,
                        double* predicted_us, double* terms)
{
  if (!prob || !sched || !predicted_us) return ALCOP_ERR_NULL;
  if (model != 0 && model != 1) return ALCOP_ERR_UNSUPPORTED;
  int rc = check_problem(*prob);
  if (rc) return rc;
  if (sched->bm <= 0 || sched->bn <= 0 || sched->bk <= 0 || sched->wm <= 0 || sched->wn <= 0 ||
      sched->stages < 1 || sched->reg_stages < 1)
    return ALCOP_ERR_SCHED;
  ModelTerms t;
  *predicted_us = predict(*prob, *sched, model, Device(), &t);
  if (terms) {
    terms[0] = t.t_kernel;
    terms[1] = t.t_threadblk;
    terms[2] = t.t_init;
    terms[3] = t.t_main_loop;
    terms[4] = t.t_epilogue;
    terms[5] = t.t_smem_load;
    terms[6] = t.t_smem_use;
    terms[7] = t.n_threadblk_batch;
  }
  return ALCOP_OK;
}

int alcop_corrector_features(const alcop_problem* prob, const alcop_sched* sched, double* x)
{
  if (!prob || !sched || !x) return ALCOP_ERR_NULL;
  int rc = check_problem(*prob);
  if (rc) return rc;
  const Device dev;
  Corrector::features(*prob, *sched, dev, x);
  return ALCOP_OK;
}

int alcop_corrector_fit(const double* x, const double* measured_us, int n, double* weights)
{
  if (!weights || (n > 0 && (!x || !measured_us))) return ALCOP_ERR_NULL;
  if (n < 0) return ALCOP_ERR_SHAPE;
  Corrector corr;
  for (int t = 0; t < n; t++) {
    if (!(measured_us[t] > 0.0)) return ALCOP_ERR_SHAPE;
    corr.add(x + (size_t)t * Corrector::D, measured_us[t]);
  }
  if (n > 0) corr.fit();
  for (int i = 0; i < Corrector::D; i++) weights[i] = corr.weight(i);
  return ALCOP_OK;
}

int alcop_time(const alcop_problem* prob, const void* A, const void* B, void* C, long lda, long ldb,
               long ldc, long strideA, long strideB, long strideC, const int* conv,
               const alcop_sched* sched, int warmup, int iters, double* mean_us, void* hip_stream)
{
  if (!sched || !mean_us) return ALCOP_ERR_NULL;
  if (iters <= 0 || warmup < 0) return ALCOP_ERR_SHAPE;
  Call c;
  int rc = call_of_problem(prob, A, B, C, lda, ldb, ldc, strideA, strideB, strideC, conv, &c);
  if (rc) return rc;
  rc = check_call(c);
  if (rc) return rc;
  const KernelEntry* e = nullptr;
  rc = check_sched(problem_of(c), *sched, &e);
  if (rc) return rc;
  rc = span_check(c, *sched);
  if (rc) return rc;
  rc = call_feasible(c, *sched, e);
  if (rc) return rc;
  return time_sched(c, *sched, e, warmup, iters, (hipStream_t)hip_stream, mean_us);
}

int alcop_tune(const alcop_problem* prob, const void* A, const void* B, void* C, long lda, long ldb,
               long ldc, long strideA, long strideB, long strideC, const int* conv, int top_k,
               int model, int variants, int iters, alcop_sched* best, double* best_us, int* trials_run,
               int* space_size, alcop_sched* log_sched, double* log_pred_us, double* log_meas_us,
               int log_cap, void* hip_stream)
{
  if (!best || !best_us) return ALCOP_ERR_NULL;
  if (top_k < 0 || iters <= 0 || model < 0 || model > 3) return ALCOP_ERR_SHAPE;
  Call c;
  int rc = call_of_problem(prob, A, B, C, lda, ldb, ldc, strideA, strideB, strideC, conv, &c);
  if (rc) return rc;
  rc = check_call(c);
  if (rc) return rc;
  const alcop_problem p = problem_of(c);
  struct Cand {
    alcop_sched s;
    const KernelEntry* e;
    double pred;
    double x[Corrector::D];
    bool tried;
  };
  std::vector<Cand> cands;
  const Device dev;
  for (const alcop_sched& s : space_of(p, 0, variants ? 1 : 0)) {
    const KernelEntry* e = nullptr;
    if (check_sched(p, s, &e) != ALCOP_OK || span_check(c, s) != ALCOP_OK ||
        call_feasible(c, s, e) != ALCOP_OK)
      continue;   // pruned
    Cand cd;
    cd.s = s;
    cd.e = e;
    cd.pred = model == 3 ? (double)cands.size() : predict(p, s, model == 2 ? 0 : model, dev, nullptr);
    cd.tried = false;
    Corrector::features(p, s, dev, cd.x);
    cands.push_back(cd);
  }
  if (space_size) *space_size = (int)cands.size();
  if (cands.empty()) return ALCOP_ERR_SCHED;
  std::stable_sort(cands.begin(), cands.end(),
                   [](const Cand& a, const Cand& b) { return a.pred < b.pred; });
  if (model == 0 || model == 1) spread_over_tiles(cands, top_k);
  const int n = top_k == 0 ? (int)cands.size() : std::min(top_k, (int)cands.size());
  Corrector corr;
  bool have = false;
  int done = 0;
  for (int t = 0; t < n; t++) {
    // next trial: models 0, 1, 3 walk their fixed ranking; model 2 takes the untried schedule
    // with the lowest corrected prediction (equal to the analytical ranking until data arrives)
    int pick = -1;
    if (model == 2) {
      double bestp = 0;
      for (int i = 0; i < (int)cands.size(); i++) {
        if (cands[i].tried) continue;
        const double pl = corr.predict_log(cands[i].x);
        if (pick < 0 || pl < bestp) {
          pick = i;
          bestp = pl;
        }
      }
    } else {
      pick = t;
    }
    double us = 0;
    rc = time_sched(c, cands[pick].s, cands[pick].e, 3, iters, (hipStream_t)hip_stream, &us);
    if (rc) return rc;
    cands[pick].tried = true;
    if (model == 2) {
      corr.add(cands[pick].x, us);
      if (t >= 2) corr.fit();
    }
    if (t < log_cap) {
      if (log_sched) log_sched[t] = cands[pick].s;
      if (log_pred_us) log_pred_us[t] = cands[pick].pred;
      if (log_meas_us) log_meas_us[t] = us;
    }
    if (!have || us < *best_us) {
      *best_us = us;
      *best = cands[pick].s;
      have = true;
    }
    done++;
  }
  if (trials_run) *trials_run = done;
  std::lock_guard<std::mutex> lk(g_cache_mu);
  g_cache[key_of(p)] = *best;
  return ALCOP_OK;
}

int alcop_sched_ranked(const alcop_problem* prob, int model, int variants, int top_k, alcop_sched* out,
                       int cap)
{
  if (!prob) return ALCOP_ERR_NULL;
  const int rc = check_problem(*prob);
  if (rc) return rc;
  if (model < 0 || model > 1 || top_k < 0) return ALCOP_ERR_SHAPE;
  struct Cand {
    alcop_sched s;
    double pred;
  };
  std::vector<Cand> cands;
  const Device dev;
  for (const alcop_sched& s : space_of(*prob, 0, variants ? 1 : 0))
    if (check_sched(*prob, s, nullptr) == ALCOP_OK) cands.push_back(Cand{s, predict(*prob, s, model, dev, nullptr)});
  std::stable_sort(cands.begin(), cands.end(), [](const Cand& a, const Cand& b) { return a.pred < b.pred; });
  spread_over_tiles(cands, top_k);
  if (out)
    for (int i = 0; i < (int)cands.size() && i < cap; i++) out[i] = cands[i].s;
  return (int)cands.size();
}

int alcop_sched_variants(const alcop_problem* prob, alcop_sched* out, int cap)
{
  if (!prob) return ALCOP_ERR_NULL;
  const int rc = check_problem(*prob);
  if (rc) return rc;
  const std::vector<alcop_sched> v = space_of(*prob, 0, 2);
  if (out)
    for (int i = 0; i < (int)v.size() && i < cap; i++) out[i] = v[i];
  return (int)v.size();
}

int alcop_sched_auto(const alcop_problem* prob, alcop_sched* out)
{
  if (!prob || !out) return ALCOP_ERR_NULL;
  int rc = check_problem(*prob);
  if (rc) return rc;
  return auto_sched(*prob, out);
}

int alcop_cache_save(const char* path)
{
  if (!path) return ALCOP_ERR_NULL;
  std::FILE* f = std::fopen(path, "w");
  if (!f) return ALCOP_ERR_IO;
  int n = 0;
  {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    for (const auto& kv : g_cache) {
      const CacheKey& k = kv.first;
      const alcop_sched& s = kv.second;
      // key order: op batch M N K transB in out conv_C transA
      std::fprintf(f, "%d %d %d %d %d %d %d %d %d %d : %d %d %d %d %d %d %d %d %d %d %d\n", std::get<0>(k),
                   std::get<1>(k), std::get<2>(k), std::get<3>(k), std::get<4>(k), std::get<9>(k),
                   std::get<5>(k), std::get<6>(k), std::get<7>(k), std::get<8>(k), s.bm, s.bn, s.bk,
                   s.wm, s.wn, s.stages, s.reg_stages, s.fuse_inner, s.raster, s.l2_prefetch, s.variant);
      n++;
    }
  }
  if (std::fclose(f) != 0) return ALCOP_ERR_IO;
  return n;
}

int alcop_cache_load(const char* path)
{
  if (!path) return ALCOP_ERR_NULL;
  return load_cache_file(path);
}

}  // extern "C"

namespace alcop {
namespace {
int load_cache_file(const char* path)
{
  std::FILE* f = std::fopen(path, "r");
  if (!f) return ALCOP_ERR_IO;
  int n = 0;
  char line[512];
  while (std::fgets(line, sizeof(line), f)) {
    int op, batch, M, N, K, tA, tB, in, out, cc;
    alcop_sched s;
    s.variant = 0;   // absent in files written before the field existed
    if (std::sscanf(line, "%d %d %d %d %d %d %d %d %d %d : %d %d %d %d %d %d %d %d %d %d %d", &op, &batch,
                    &M, &N, &K, &tA, &tB, &in, &out, &cc, &s.bm, &s.bn, &s.bk, &s.wm, &s.wn,
                    &s.stages, &s.reg_stages, &s.fuse_inner, &s.raster, &s.l2_prefetch,
                    &s.variant) < 20)
      continue;
    alcop_problem p;
    p.op = (alcop_op)op;
    p.batch = batch;
    p.M = M;
    p.N = N;
    p.K = K;
    p.transA = tA;
    p.transB = tB;
    p.in = (alcop_dtype)in;
    p.out = (alcop_dtype)out;
    p.conv_C = cc;
    if (check_sched(p, s, nullptr) != ALCOP_OK) continue;   // not runnable here: ignore the entry
    std::lock_guard<std::mutex> lk(g_cache_mu);
    g_cache[key_of(p)] = s;
    n++;
  }
  std::fclose(f);
  return n;
}
}  // namespace
}  // namespace alcop

extern "C" {

const char* alcop_strerror(int code)
{
  switch (code) {
    case ALCOP_OK: return "ok";
    case ALCOP_ERR_NULL: return "null pointer";
    case ALCOP_ERR_DTYPE: return "unsupported element type";
    case ALCOP_ERR_ALIGN: return "pointer, leading dimension or stride not aligned";
    case ALCOP_ERR_SHAPE: return "bad shape (size <= 0, K or N not a multiple of 8, conv C not a multiple of 8)";
    case ALCOP_ERR_SCHED: return "schedule not built or infeasible";
    case ALCOP_ERR_LAUNCH: return "HIP launch failed";
    case ALCOP_ERR_UNSUPPORTED: return "not supported";
    case ALCOP_ERR_SIZE: return "operand spans 2 GiB or more";
    case ALCOP_ERR_IO: return "cache file could not be opened, read or written";
    default: return "unknown status";
  }
}

const char* alcop_version(void) { return "alcop-mi355x 0.1 (gfx950)"; }

}  // extern "C"
