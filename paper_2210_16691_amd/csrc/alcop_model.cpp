// Static latency model (paper Sec. 5).  Symbols follow Table 1; where the paper leaves a term
// open the reading taken is stated next to it.
#include "alcop_model.h"

#include <algorithm>
#include <cmath>

namespace alcop {

// Table 1, "Pipeline Latency Model".  A load is hidden when the work that can overlap it
// (the other N_pipe-1 stages of this worker plus N_mplx-1 other workers) lasts at least as
// long; otherwise every N_pipe iterations cost one exposed load plus one use.
double pipeline_latency(double t_load, double t_use, double n_loop, double n_pipe, double n_mplx)
{
  if (t_load <= (n_pipe * n_mplx - 1.0) * t_use) return t_use * n_loop;
  return (t_load + t_use) * n_loop / n_pipe;
}

static double ceil_div(double a, double b) { return std::ceil(a / b); }

double predict(const alcop_problem& prob, const alcop_sched& s, int model, const Device& dev,
               ModelTerms* terms)
{
  const double bm = s.bm, bn = s.bn, bk = s.bk, wm = s.wm, wn = s.wn;
  const double S = s.stages, R = s.reg_stages;
  const double out_bytes = prob.out == ALCOP_F32 ? 4.0 : 2.0;
  const double batch = prob.batch > 0 ? prob.batch : 1;
  const double ntm = ceil_div(prob.M, bm), ntn = ceil_div(prob.N, bn);
  const double tiles = ntm * ntn;
  const double n_blocks = tiles * batch;
  const double n_warp = (bm / wm) * (bn / wn);              // N_warp_per_threadblk
  const double n_smem_loop = std::ceil(prob.K / bk);        // N_smem_loop (a partial tile counts)
  const double n_reg_loop = bk / 16.0;                       // N_reg_loop (MFMA k = 16)
  // Schedule variant 1 of a convolution keeps the input patch of the tile in LDS: the A rows are
  // loaded once per block, not once per filter tap, so a k-tile brings in 1/taps of them, and
  // the patch (reading: tile plus half a tile of halo) occupies LDS beside the ring of B tiles.
  const bool patch = prob.op == ALCOP_OP_CONV2D && s.variant == 1 && prob.conv_C > 0;
  const double taps = patch ? std::max(1.0, (double)prob.K / prob.conv_C) : 1.0;
  const double a_rows = bm / taps;                           // A rows fetched per k-tile
  const double stage_bytes = (a_rows + bn) * bk * 2.0;      // Bytes_one_smem_loop
  // Schedule variant 2: persistent blocks of four consumer and four producer waves; the ring is
  // followed by a staging band per consumer wave, and at most two blocks share a compute unit.
  const bool persistent = s.variant == 2;
  const double lds_use = patch ? S * bn * bk * 2.0 + 1.5 * bm * bk * 2.0
                               : S * stage_bytes + (persistent ? n_warp * 32.0 * (wn * 4.0 + 16.0) : 0.0);
  const double frag_bytes = n_warp * (wm + wn) * 16.0 * 2.0; // Bytes_one_reg_loop (LDS reads)
  const double flops_reg_loop = 2.0 * bm * bn * 16.0;        // FLOPs_one_reg_loop

  if (model == 1) {
    // Bottleneck-only model (Sec. 6.4): full utilisation of every resource, no latency terms.
    const double t_cmp = n_blocks * n_smem_loop * n_reg_loop * flops_reg_loop /
                         (dev.num_cu * dev.flop_per_us_cu);
    const double t_lds = n_blocks * n_smem_loop * n_reg_loop * frag_bytes /
                         (dev.num_cu * dev.bw_lds_cu);
    const double t_mem = (n_blocks * n_smem_loop * stage_bytes + n_blocks * bm * bn * out_bytes) /
                         dev.bw_dram;
    const double t = std::max(t_cmp, std::max(t_lds, t_mem));
    if (terms) *terms = ModelTerms{t, t, 0, t, 0, t_mem, t_cmp, 1};
    return t;
  }

  // --- simulated block scheduler (Sec. 5.1: blocks per SM limited by shared memory and
  // registers).  Reading: registers per lane = accumulators + R fragment sets + 48.
  const double regs = wm * wn / 64.0 + R * (wm / 32.0 + wn / 32.0) * 4.0 + 48.0;
  const double waves_per_simd = std::max(1.0, std::min(8.0, std::floor(dev.regs_per_lane / regs)));
  double blk_per_cu = std::min(std::floor(dev.lds_bytes / lds_use),
                               std::floor(waves_per_simd * dev.simd_per_cu / n_warp));
  blk_per_cu = std::max(1.0, blk_per_cu);
  if (persistent) blk_per_cu = std::max(1.0, std::min(2.0, std::floor(dev.lds_bytes / lds_use)));
  blk_per_cu = std::min(blk_per_cu, ceil_div(n_blocks, dev.num_cu));   // no more than exist
  const double slots = dev.num_cu * blk_per_cu;
  const double n_batch = ceil_div(n_blocks, slots);           // N_threadblk_batch
  const double n_in_batch = std::min(n_blocks, slots);        // N_threadblk_per_threadblk_batch

  // --- computation latency.  Reading of Util(N_warp, N_blk): the share of one CU's matrix
  // throughput that ONE block obtains: all pipes busy once N_warp*N_blk >= 4, split evenly
  // among the co-resident blocks.
  const double util = std::min(1.0, n_warp * blk_per_cu / dev.simd_per_cu) / blk_per_cu;
  const double t_compute = flops_reg_loop / (dev.flop_per_us_cu * util);

  // --- register-level loop.  T_reg_load is not printed in the paper; reading: same form as the
  // LLC term, latency + bytes / bandwidth, the LDS port shared by the co-resident blocks.
  const double t_reg_load = dev.lat_lds + frag_bytes * blk_per_cu / dev.bw_lds_cu;
  // Deliberate deviation from Table 1, which gives N_warp_per_threadblk as the multiplexing
  // factor of the inner pipeline: a wavefront is pinned to one of the CU's four SIMDs, and only
  // wavefronts of the same SIMD can fill each other's load latency, so the factor is the number
  // of wavefronts per SIMD (four waves on four SIMDs do not multiplex at all).
  const double mplx_inner = std::max(1.0, n_warp * blk_per_cu / dev.simd_per_cu);
  double t_smem_use = pipeline_latency(t_reg_load, t_compute, n_reg_loop, R, mplx_inner);
  // The paper's T_smem_use is the fused steady state.  Without fusion the register pipeline is
  // refilled in every outer iteration: one exposed fragment load per ko.
  if (!s.fuse_inner && s.reg_stages >= 2) t_smem_use += t_reg_load;
  // LDS port occupancy (not in Table 1): the LDS serves the fragment reads of every wave and
  // the direct-to-LDS writes of the incoming k-tile through one port.  The K-contiguous operand
  // is read at bw_lds, the N-contiguous one through the transposing read at its own rate.  However well
  // latencies are hidden, a k-tile cannot be consumed faster than the port moves its bytes.
  {
    const double a_read = bm * bk * 2.0 * (bn / wn);   // every A row is read by the waves along n
    const double b_read = bn * bk * 2.0 * (bm / wm);
    const double t_port = (a_read / (prob.transA ? dev.bw_lds_tr_cu : dev.bw_lds_cu) +
                           b_read / (prob.transB ? dev.bw_lds_cu : dev.bw_lds_tr_cu) +
                           stage_bytes / dev.bw_lds_cu) * blk_per_cu;
    t_smem_use = std::max(t_smem_use, t_port);
    // Fill path (not in Table 1 either): the pipeline criterion treats a load as a latency to
    // hide, but one compute unit's L2 -> LDS path delivers only bw_llc / num_cu bytes per
    // microsecond; the blocks of a CU cannot consume k-tiles faster than it delivers them.
    const double t_fill = stage_bytes * blk_per_cu / (dev.bw_llc / dev.num_cu);
    t_smem_use = std::max(t_smem_use, t_fill);
  }

  // --- memory latency
  const double t_llc = dev.lat_llc + stage_bytes * n_in_batch / dev.bw_llc;
  // DRAM working set of a block batch: the co-resident blocks of one matrix form a near-square
  // patch of tiles; distinct row panels and column panels are fetched once.
  const double per_mat = std::min(tiles, n_in_batch);
  const double mats = ceil_div(n_in_batch, tiles);
  const double rows_u = std::min(ntm, std::ceil(std::sqrt(per_mat)));
  const double cols_u = std::min(ntn, ceil_div(per_mat, rows_u));
  const double workset = (rows_u * a_rows + cols_u * bn) * bk * 2.0 * mats;
  const double t_dram = dev.lat_dram + workset / dev.bw_dram;
  const double t_smem_load = std::max(t_llc, t_dram);

  const double t_init = t_smem_load + t_reg_load;
  if (persistent) {
    // Schedule variant 2 (not in the paper; its model applied to the kernel's loop structure):
    // a block's tiles form ONE load-and-use loop of tiles_per_block * N_smem_loop iterations; the
    // epilogue of a tile is consumer work inside that loop (its stores are not waited for, so only
    // their bandwidth term counts, spread over the tile's iterations); T_init is paid once and one
    // write latency ends the kernel.
    const double tiles_per_block = ceil_div(n_blocks, slots);
    const double t_store = bm * bn * out_bytes * n_in_batch / dev.bw_dram_write;
    const double t_use = t_smem_use + t_store / n_smem_loop;
    const double t_main = pipeline_latency(t_smem_load, t_use, tiles_per_block * n_smem_loop, S, blk_per_cu);
    const double t_kernel = t_init + t_main + dev.lat_dram_write;
    if (terms)
      *terms = ModelTerms{t_kernel, t_kernel, t_init, t_main, dev.lat_dram_write, t_smem_load, t_use, 1.0};
    return t_kernel;
  }
  const double t_main = pipeline_latency(t_smem_load, t_smem_use, n_smem_loop, S, blk_per_cu);
  const double t_epi = dev.lat_dram_write + bm * bn * out_bytes * n_in_batch / dev.bw_dram_write;
  const double t_blk = t_init + t_main + t_epi;
  const double t_kernel = t_blk * n_batch;
  if (terms)
    *terms = ModelTerms{t_kernel, t_blk, t_init, t_main, t_epi, t_smem_load, t_smem_use, n_batch};
  return t_kernel;
}

// ---- measurement-corrected model ------------------------------------------------------------
Corrector::Corrector() : n_(0)
{
  for (int i = 0; i < D; i++) {
    xty_[i] = 0;
    prior_[i] = 0;
    for (int j = 0; j < D; j++) xtx_[i][j] = 0;
  }
  prior_[1] = 1.0;   // log t = 1 * log(analytical prediction)
  for (int i = 0; i < D; i++) w_[i] = prior_[i];
}

void Corrector::features(const alcop_problem& prob, const alcop_sched& s, const Device& dev,
                         double* x)
{
  const double waves = (double)(s.bm / s.wm) * (s.bn / s.wn);
  x[0] = 1.0;
  x[1] = std::log(predict(prob, s, 0, dev, nullptr));
  x[2] = std::log(predict(prob, s, 1, dev, nullptr));
  x[3] = std::log2((double)s.bm * s.bn) - 14.0;     // tile area relative to 128 x 128
  x[4] = std::log2((double)s.bk) - 6.0;
  x[5] = s.stages - 2.0;
  x[6] = s.reg_stages - 1.0;
  x[7] = s.fuse_inner ? 1.0 : 0.0;
  x[8] = std::log2(waves) - 2.0;
  x[9] = s.l2_prefetch > 0 ? 1.0 : 0.0;
}

void Corrector::add(const double* x, double measured_us)
{
  const double y = std::log(measured_us);
  for (int i = 0; i < D; i++) {
    xty_[i] += x[i] * y;
    for (int j = 0; j < D; j++) xtx_[i][j] += x[i] * x[j];
  }
  n_++;
}

void Corrector::fit()
{
  // minimise sum (y - w.x)^2 + lambda |w - prior|^2 : (XtX + lambda I) w = Xty + lambda prior
  const double lambda = 0.3;
  double a[D][D + 1];
  for (int i = 0; i < D; i++) {
    for (int j = 0; j < D; j++) a[i][j] = xtx_[i][j] + (i == j ? lambda : 0.0);
    a[i][D] = xty_[i] + lambda * prior_[i];
  }
  for (int c = 0; c < D; c++) {            // Gaussian elimination with partial pivoting
    int piv = c;
    for (int r = c + 1; r < D; r++)
      if (std::fabs(a[r][c]) > std::fabs(a[piv][c])) piv = r;
    if (std::fabs(a[piv][c]) < 1e-12) return;   // singular: keep the previous weights
    if (piv != c)
      for (int j = 0; j <= D; j++) std::swap(a[c][j], a[piv][j]);
    for (int r = 0; r < D; r++) {
      if (r == c) continue;
      const double f = a[r][c] / a[c][c];
      for (int j = c; j <= D; j++) a[r][j] -= f * a[c][j];
    }
  }
  for (int i = 0; i < D; i++) w_[i] = a[i][D] / a[i][i];
}

double Corrector::predict_log(const double* x) const
{
  double y = 0;
  for (int i = 0; i < D; i++) y += w_[i] * x[i];
  return y;
}

}  // namespace alcop
