// Static latency model of a schedule (paper Sec. 5, Table 1), host code, fp64.
#pragma once
#include "../../include/alcop.h"

namespace alcop {

// Machine constants of the model (the LAT_* / BW_* / Throughput symbols of Table 1).
// Times in microseconds, sizes in bytes, rates per microsecond.
struct Device {
  int num_cu = 256;                 // compute units ("SMs")
  int simd_per_cu = 4;              // matrix pipes per CU
  double lds_bytes = 163840.0;      // LDS per CU
  double regs_per_lane = 512.0;     // VGPR + AGPR budget per SIMD lane
  // dense fp16/bf16 MFMA: 4096 flop/clk/CU; the clock a GEMM sustains under the power cap is
  // about 1.8 GHz (measured inside the kernel), not the 2.4 GHz peak
  double clk_per_us = 1800.0;
  double flop_per_us_cu = 4096.0 * 1800.0;
  double lat_lds = 128.0 / 1800.0;
  // LDS read rates measured with enough waves in flight to hide the latency: ds_read_b128
  // 256 B/clk per CU (4 clk per wave instruction), ds_read_b64_tr_b16 ~170 B/clk (3 clk per wave
  // instruction of 512 bytes); direct-to-LDS writes are taken at the b128 rate
  double bw_lds_cu = 256.0 * 1800.0;
  double bw_lds_tr_cu = 170.0 * 1800.0;
  // L2 / Infinity Cache -> LDS, aggregate: a CU's direct-to-LDS fill path delivers ~56 B/clk alone
  // and ~40 B/clk when all 256 stream (8 L2s near their bandwidth, ~20 % of the requests missing)
  double lat_llc = 0.6, bw_llc = 40.0 * 256.0 * 1800.0;
  double lat_dram = 1.2, bw_dram = 8.0e6;     // HBM3E read
  double lat_dram_write = 1.0, bw_dram_write = 8.0e6;
};

struct ModelTerms {
  double t_kernel, t_threadblk, t_init, t_main_loop, t_epilogue, t_smem_load, t_smem_use,
      n_threadblk_batch;
};

// The pipeline latency model of Table 1, second row.
double pipeline_latency(double t_load, double t_use, double n_loop, double n_pipe, double n_mplx);

// model 0: pipeline-aware model of Table 1; model 1: bottleneck-only comparison model (Sec. 6.4).
// Returns predicted microseconds; fills terms if not null.
double predict(const alcop_problem& prob, const alcop_sched& s, int model, const Device& dev,
               ModelTerms* terms);

// Measurement-corrected cost model (paper Sec. 5.3, "Analytical + ML": a learned cost model that
// starts from the analytical predictions and is updated with profiled trials).  The learner is
// a ridge regression on log-time whose prior is the analytical model itself: with no
// measurements it ranks exactly like model 0; every timed trial pulls the weights of a few
// schedule features (tile area, k-tile, stages, waves, fusion, L2 touches) towards what was
// measured on this machine and shape.
class Corrector {
 public:
  static constexpr int D = 10;
  Corrector();
  static void features(const alcop_problem& prob, const alcop_sched& s, const Device& dev,
                       double* x /* D */);
  void add(const double* x, double measured_us);   // one profiled trial
  void fit();                                      // ridge solve towards the prior
  double predict_log(const double* x) const;       // log(predicted microseconds)
  double weight(int i) const { return w_[i]; }

 private:
  double xtx_[D][D], xty_[D], w_[D], prior_[D];
  int n_;
};

}  // namespace alcop
