/*
 * alcop_diag.h - C ABI of libalcop_diag.so, a measurement aid that ships beside libalcop.so.
 *
 * Where does the time of the pipelined main loop go?  The library holds a few instances of the
 * very same kernel template as libalcop.so, each compiled once per "ablation": a hardware-policy
 * class derived from the gfx950 one that leaves out ONE class of operation (the direct-to-LDS
 * loads, the LDS -> register reads, the matrix instructions, the block barrier, the stores of C).  The loop, its
 * addresses, its bounds and its launch shape are those of the product kernel; an ablated kernel
 * only does less, so every access it makes is one the full kernel makes too.  Its OUTPUT IS
 * WRONG by construction; only its time means something.  Timing is by HIP events around
 * back-to-back launches; no kernel writes anything but C.
 *
 * This is the evidence behind the statements about load / compute overlap (paper Sec. 1, Fig. 2:
 * what pipelining hides) and about which resource bounds a schedule (Sec. 5, Table 1).
 */
#ifndef ALCOP_DIAG_H
#define ALCOP_DIAG_H
#ifdef __cplusplus
extern "C" {
#endif

/* which operations a variant drops (bit mask) */
enum {
  ALCOP_DIAG_FULL = 0,
  ALCOP_DIAG_NO_DMA = 1,      /* no direct-to-LDS loads: the ring keeps what LDS happened to hold */
  ALCOP_DIAG_NO_LDS_READ = 2, /* no fragment reads: the matrix cores consume undefined registers */
  ALCOP_DIAG_NO_MFMA = 4,     /* no matrix instructions                                          */
  ALCOP_DIAG_NO_BARRIER = 8,  /* no block-wide barrier (waits on the counters stay)              */
  ALCOP_DIAG_NO_STORE = 16,   /* no global stores of C (conversion and LDS staging stay)         */
  ALCOP_DIAG_NO_SWIZZLE = 32, /* LDS tile images not permuted: every operation stays and the    */
                              /* result is right, but the fragment reads meet bank conflicts    */
  ALCOP_DIAG_COPY = 64        /* nothing dropped: a second, separately named copy of the full   */
                              /* kernel, so that a profiler keeps runs on other operands (all   */
                              /* zeros, say) apart from the runs of variant 0                   */
};

/* Number of kernel configurations built in, and a description of configuration i
 * ("f16 128x128x64 w64x64 S4 R2 F1"), NULL if i is out of range. */
int alcop_diag_configs(void);
const char* alcop_diag_config_name(int i);

/*
 * Times configuration `config` with the operations in `drop` left out: C (fp16 / bf16 as the
 * configuration says, row-major M x N) = A (M x K, row-major) . B (K x N, row-major), all DEVICE
 * pointers owned by the caller, 16-byte aligned, M, N multiples of the tile and K of the k-tile.
 * `iters` back-to-back launches after 20 warm-up launches, 3 repeats; writes the best mean
 * microseconds per launch.  Only the combinations 0, 1, 2, 4, 8, 16, 1|2, 2|4, 1|2|4 (what is
 * left is launch, prologue, barriers and epilogue), 1|2|4|16, 32 and 64 are built.
 * Returns 0, or -1 (bad argument / combination not built), -2 (HIP error).
 */
int alcop_diag_time(int config, int drop, const void* A, const void* B, void* C, int M, int N,
                    int K, int iters, double* mean_us /* host */);

/*
 * Microseconds per launch of a kernel that does nothing (`blocks` x `threads`, 1..65536 x 1..1024),
 * `iters` back-to-back launches on the default stream after 20 warm-up launches, best of 3
 * repeats: the floor under every per-launch time this library reports.
 * Returns 0, or -1 (bad argument), -2 (HIP error).
 */
int alcop_diag_launch_floor(int blocks, int threads, int iters, double* mean_us /* host */);

#ifdef __cplusplus
}
#endif
#endif
