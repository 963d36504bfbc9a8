/*
 * alcop.h - C ABI of the MI355X (gfx950) load-compute-pipelined tensor kernels.
 *
 * The library implements the tiled main loop that the ALCOP paper (arXiv 2210.16691)
 * pipelines, for the three operators the paper names as pipelinable (Sec. 6.2: MatMul,
 * batched MatMul, Conv2D; half-precision inputs on the matrix cores, Sec. 6.1):
 *
 *   - tiles of A and B travel HBM -> LDS through an S-slot circular buffer filled by
 *     asynchronous direct-to-LDS loads (Sec. 4.2, transformation steps 1-5: buffer
 *     expansion, index shift by S-1, slot = iteration mod S, prologue of S-1 loads,
 *     producer/consumer synchronisation);
 *   - fragments travel LDS -> registers through an R-slot register buffer (multi-level
 *     pipelining, Fig. 3(c));
 *   - with fuse_inner the register pipeline is one pipeline over all (ko, ki) steps: the
 *     first fragment of tile ko+1 is fetched during the last step of tile ko (inner-pipeline
 *     fusion, Fig. 3(d) and Sec. 4.1 step 5);
 *   - a static latency model ranks schedules without running them and a tuner times only the
 *     best-ranked ones (Sec. 5, Table 1 and Sec. 5.3).
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library never
 *     allocates, frees or copies device memory (the split-K entry points take their scratch
 *     memory as a workspace argument).  Host pointers are marked "host".
 *   - Calls enqueue work on the given HIP stream (a hipStream_t passed as void*; NULL is the
 *     default stream) and return without synchronising.  alcop_tune, alcop_tune_splitk and
 *     alcop_time are the exceptions: they synchronise the stream in order to time launches.
 *   - Return value: ALCOP_OK (0) or a negative alcop_status.  Nothing is launched when an
 *     error is returned.  No entry point throws or aborts.
 *   - Element types: inputs are IEEE binary16 (ALCOP_F16) or bfloat16 (ALCOP_BF16); products
 *     are accumulated in fp32 on the matrix cores in a fixed order (ko ascending, ki
 *     ascending), so for a fixed tile shape the result does not depend on stages,
 *     reg_stages or fuse_inner.  The output is the fp32 accumulator converted with
 *     round-to-nearest-even to ALCOP_F16 / ALCOP_BF16, or stored as is (ALCOP_F32).
 *   - Alignment: every tensor base pointer is 16-byte aligned; leading dimensions and batch
 *     strides are multiples of 8 elements.
 *   - Shapes: K and N must be multiples of 8; M is free.  Edge tiles in M, N and K are loaded
 *     with zero fill and stored under a mask (convolution: C must be a multiple of 8).  Each
 *     operand of one GEMM (one batch entry) must span less than 2 GiB.
 */
#ifndef ALCOP_H
#define ALCOP_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { ALCOP_F16 = 0, ALCOP_BF16 = 1, ALCOP_F32 = 2 /* output only */ } alcop_dtype;

typedef enum {
  ALCOP_OK = 0,
  ALCOP_ERR_NULL = -1,        /* a required pointer is NULL                                  */
  ALCOP_ERR_DTYPE = -2,       /* unsupported input / output element type                     */
  ALCOP_ERR_ALIGN = -3,       /* pointer, leading dimension or stride not aligned as stated  */
  ALCOP_ERR_SHAPE = -4,       /* non-positive size, K or N (conv: C) not a multiple of 8     */
  ALCOP_ERR_SCHED = -5,       /* schedule infeasible: no such kernel, LDS or wait-counter    */
                              /* limit exceeded, fuse_inner without reg_stages=2/stages>=2   */
  ALCOP_ERR_LAUNCH = -6,      /* the HIP runtime refused the launch                          */
  ALCOP_ERR_UNSUPPORTED = -7, /* valid request outside what is built (e.g. an unknown act)   */
  ALCOP_ERR_SIZE = -8,        /* an operand spans 2 GiB or more; a workspace is too small    */
  ALCOP_ERR_IO = -9           /* a cache file could not be opened, read or written           */
} alcop_status;

/*
 * Schedule parameters: the knobs the paper's tuner searches (tile sizes and per-buffer
 * stage counts, Sec. 4.1 step 1 and Sec. 6.1).  A NULL schedule pointer, or bm == 0, asks
 * the library to pick: the schedule a tuning run left in the cache for this problem, else the
 * entry with the lowest predicted latency under the static model among the feasible kernels
 * of the default space.
 */
typedef struct {
  int bm, bn, bk;     /* block tile of C (bm x bn) and reduction step bk                    */
  int wm, wn;         /* per-wavefront tile; the block runs (bm/wm)*(bn/wn) wavefronts      */
  int stages;         /* S: LDS ring depth, 1..4; 1 = load and use strictly alternate       */
  int reg_stages;     /* R: 1 = fragment loaded then used; 2 = next fragment prefetched;    */
                      /* 3, 4 = R-1 fragments in flight (fused only, (R-1)*16 <= bk)        */
  int fuse_inner;     /* 1 = register pipeline runs across ko (needs R>=2 and S>=2)         */
  int raster;         /* block -> tile order: 0 row-major, 1 XCD-grouped panels             */
  int l2_prefetch;    /* third buffer level (HBM -> L2): lines of k-tile kt+l2_prefetch are  */
                      /* touched when k-tile kt is issued; 0 = off; needs raster = 1         */
  int variant;        /* 0 = the default kernel.  Convolution only, 1 = input patch resident */
                      /* in LDS: the block loads its output tile's input pixels plus halo    */
                      /* once and forms the filter taps by shifted LDS reads, so only the    */
                      /* weights stream through the ring.  Needs stride 1, RSCK weights,     */
                      /* bk equal to the channel count, and a patch that fits the LDS;       */
                      /* a call that does not meet this returns ALCOP_ERR_SCHED.             */
                      /* 2 = persistent producer / consumer kernel (any operator): a block    */
                      /* stays on its compute unit and walks a list of output tiles; four     */
                      /* producer waves keep the S-stage ring filled across tile boundaries   */
                      /* while four consumer waves multiply and store, so the loads of the    */
                      /* next tile overlap the epilogue of this one (the paper's load / use   */
                      /* overlap, Sec. 1, carried across tiles; for short reduction axes,     */
                      /* Sec. 6.1).  Needs stages >= 2, reg_stages = 2 (fuse_inner 0 or 1)    */
                      /* or reg_stages = 4 with fuse_inner = 1 and bk >= 64 (three fragments   */
                      /* in flight, the barrier early in the k-tile),                           */
                      /* l2_prefetch = 0, four waves' worth of wave tiles per block tile, and */
                      /* for a convolution a k-tile that divides the channel count.  Results  */
                      /* are bit-identical to the default kernels of the same tile.  The      */
                      /* number of blocks is one or two per compute unit (by LDS), at most    */
                      /* the number of tiles; the environment variable ALCOP_STREAM_BLOCKS    */
                      /* (a positive integer, read at every launch) overrides it              */
} alcop_sched;

/* Problem description used by the model / tuner / feasibility entry points. */
typedef enum { ALCOP_OP_GEMM = 0, ALCOP_OP_BMM = 1, ALCOP_OP_CONV2D = 2 } alcop_op;
typedef struct {
  alcop_op op;
  int batch;          /* 1 for GEMM and conv                                                */
  int M, N, K;        /* GEMM view; for conv M = N_img*P*Q, N = K_out, K = R*S*C           */
  int transB;         /* 1: B stored N x K (K contiguous)                                   */
  alcop_dtype in, out;
  int conv_C;         /* conv only: input channels (bk must divide it)                      */
  int transA;         /* 1: A stored K x M (M contiguous); GEMM / BMM only                  */
} alcop_problem;

/*
 * C[M,N] = A[M,K] . B[K,N]        (paper Sec. 6.1 "MatMul")
 *   A: transA == 0: row-major M x K, lda >= K;  transA == 1: stored K x M, lda >= M
 *      (M must then be a multiple of 8).
 *   B: transB == 0: row-major K x N, ldb >= N;  transB == 1: stored N x K, ldb >= K.
 *   C: row-major M x N, ldc >= N, element type `out`.
 */
int alcop_gemm(const void* A, const void* B, void* C, int M, int N, int K,
               long lda, long ldb, long ldc, int transA, int transB,
               alcop_dtype in, alcop_dtype out, const alcop_sched* sched /* host */,
               void* hip_stream);

/*
 * Batched matmul (paper Sec. 6.1 "BMM"; attention Q.K^T uses transB = 1, P.V transB = 0).
 * Batch entry b uses A + b*strideA, B + b*strideB, C + b*strideC (strides in elements).
 */
int alcop_bmm(const void* A, const void* B, void* C, int batch, int M, int N, int K,
              long lda, long ldb, long ldc, long strideA, long strideB, long strideC,
              int transA, int transB, alcop_dtype in, alcop_dtype out,
              const alcop_sched* sched /* host */, void* hip_stream);

/*
 * GEMM / batched matmul with an elementwise function fused on the consumer side
 * (paper Sec. 3.2, "Fusion": an elementwise f(.) is folded into the operator that consumes the
 * data instead of into the copy that fills a pipelined buffer, so the buffer is still produced
 * by an asynchronous copy and stays pipelinable).  Here f is applied to the fp32 accumulators in
 * the epilogue, before the conversion to the output type:
 *     C[i][j] = act( alpha * sum_k A(i,k) B(k,j) + bias[j] )
 * alpha: host scalar (e.g. 1/sqrt(d) for attention scores); bias: DEVICE pointer to N fp32
 * values, 16-byte aligned, or NULL; act: 0 = identity, 1 = ReLU.  ep == NULL means
 * alpha = 1, no bias, identity.  For alcop_bmm_fused the same bias vector is used by every batch.
 */
typedef struct {
  float alpha;
  const void* bias;
  int act;
} alcop_epilogue;

int alcop_gemm_fused(const void* A, const void* B, void* C, int M, int N, int K,
                     long lda, long ldb, long ldc, int transA, int transB,
                     alcop_dtype in, alcop_dtype out, const alcop_epilogue* ep /* host */,
                     const alcop_sched* sched /* host */, void* hip_stream);

int alcop_bmm_fused(const void* A, const void* B, void* C, int batch, int M, int N, int K,
                    long lda, long ldb, long ldc, long strideA, long strideB, long strideC,
                    int transA, int transB, alcop_dtype in, alcop_dtype out,
                    const alcop_epilogue* ep /* host */, const alcop_sched* sched /* host */,
                    void* hip_stream);

/*
 * 2-D convolution as an implicit GEMM (paper Sec. 6.2 "Conv2D": its reduction loop over
 * (r, s, c) is a sequential load-and-use loop in the sense of Sec. 3.1, rule 2).
 *   x: NHWC  [N][H][W][C];  w: RSCK [R][S][C][K];  y: NPQK [N][P][Q][K],
 *   P = (H + 2*pad_h - R)/stride_h + 1, Q likewise.  Cross-correlation, zero padding,
 *   dilation 1, one group.  GEMM view: M = N*P*Q, N = K, reduction = R*S*C in (r,s,c) order.
 *   C and K must be multiples of 8; x must span < 2 GiB.  When the schedule's bk divides C a
 *   k-tile lies inside one filter tap and the tap is tracked once per wave; otherwise (C = 8, 24,
 *   40, ... or bk = 64 with C = 96) every lane tracks the tap of its own 8-channel chunk.  The
 *   library holds kernels of both kinds; which one a schedule means follows from C and bk.
 */
int alcop_conv2d_igemm(const void* x, const void* w, void* y, int N, int H, int W, int C,
                       int K, int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                       alcop_dtype in, alcop_dtype out, const alcop_sched* sched /* host */,
                       void* hip_stream);

/*
 * The same convolution with the weights stored KRSC, [K][R][S][C]: the filter index outermost,
 * i.e. B of the GEMM view stored N x (R*S*C) with the reduction axis contiguous (both operand
 * tiles are then read from LDS with plain 16-byte reads).  In an alcop_problem this layout is
 * op = ALCOP_OP_CONV2D with transB = 1.  Everything else as for alcop_conv2d_igemm.
 */
int alcop_conv2d_igemm_krsc(const void* x, const void* w, void* y, int N, int H, int W, int C,
                            int K, int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                            alcop_dtype in, alcop_dtype out, const alcop_sched* sched /* host */,
                            void* hip_stream);

/*
 * Convolution with the consumer-side elementwise function of alcop_gemm_fused on the
 * accumulators: y[n][p][q][k] = act(alpha * conv(x, w) + bias[k]) - the convolution + bias + ReLU
 * layer of the paper's ResNet / VGG models in one kernel.  krsc = 0: weights RSCK, 1: KRSC.
 * ep == NULL means alpha = 1, no bias, identity.
 */
int alcop_conv2d_igemm_fused(const void* x, const void* w, void* y, int N, int H, int W, int C,
                             int K, int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                             alcop_dtype in, alcop_dtype out, const alcop_epilogue* ep /* host */,
                             int krsc, const alcop_sched* sched /* host */, void* hip_stream);

/*
 * Dilated convolution (beyond the paper's dilation-1 operators; the gather of Sec. 4's
 * load-and-use loop only changes its addresses): filter tap (r, s) reads
 * x[n][p*stride_h - pad_h + r*dil_h][q*stride_w - pad_w + s*dil_w][c];
 * P = (H + 2*pad_h - dil_h*(R-1) - 1)/stride_h + 1, Q likewise.  dil_h, dil_w >= 1.
 * krsc: 0 = weights [R][S][C][K], 1 = [K][R][S][C]; ep (host, may be NULL) as for
 * alcop_conv2d_igemm_fused.  Schedules as for alcop_conv2d_igemm, except that the LDS-resident
 * patch variant (variant 1) needs dilation 1.  Errors as for alcop_conv2d_igemm.
 */
int alcop_conv2d_igemm_dilated(const void* x, const void* w, void* y, int N, int H, int W, int C,
                               int K, int R, int S, int stride_h, int stride_w, int pad_h,
                               int pad_w, int dil_h, int dil_w, int krsc, alcop_dtype in,
                               alcop_dtype out, const alcop_epilogue* ep /* host, may be NULL */,
                               const alcop_sched* sched /* host */, void* hip_stream);

/*
 * Operands the pipelined loops cannot take as they are (paper Sec. 4.2: a pipeline stage is
 * filled by asynchronous copies; here they move 16-byte chunks, hence the alignment rules of
 * alcop_gemm): N or K not a multiple of 8, M not a multiple of 8 with transA, leading dimensions,
 * batch strides or base addresses that are not 16-byte aligned.  A, B (and the bias) are first
 * copied into `workspace` with every extent rounded up to 8 elements and the tails zero-filled,
 * the product is computed there by the ordinary kernels (same schedules, same k order; the extra
 * k terms are exact zeros, so every valid element equals what an aligned call on the same values
 * returns), and the valid M x N part is copied to C element by element; bytes of C outside the
 * valid elements (row padding) are not touched.  Three small copy kernels besides the product:
 * meant for odd shapes, not for speed.
 *   A, B, C: DEVICE pointers aligned to their element size; lda, ldb, ldc, strides in elements,
 *     any value allowed by the shape (lda >= K or M, ...); batch = 1 with strides 0 is a GEMM.
 *   ep: host, may be NULL; ep->bias: DEVICE pointer to N fp32 values, 4-byte aligned.
 *   sched: a schedule for the padded problem (M, N, K rounded up to 8), or NULL = the library's pick.
 *   workspace: DEVICE memory, 16-byte aligned, at least alcop_unaligned_workspace_bytes(batch, M, N,
 *     K, out) bytes (that function returns 0 for arguments no call accepts); owned by the caller,
 *     overwritten by the call.  Calls that share a workspace must be ordered on one stream.
 * Errors as for alcop_bmm; ALCOP_ERR_SIZE also if the workspace is too small.
 */
size_t alcop_unaligned_workspace_bytes(int batch, int M, int N, int K, alcop_dtype out);
int alcop_bmm_unaligned(const void* A, const void* B, void* C, int batch, int M, int N, int K,
                        long lda, long ldb, long ldc, long strideA, long strideB, long strideC,
                        int transA, int transB, alcop_dtype in, alcop_dtype out,
                        const alcop_epilogue* ep /* host, may be NULL */,
                        const alcop_sched* sched /* host */, void* workspace,
                        size_t workspace_bytes, void* hip_stream);

/*
 * The same for a convolution whose channel counts are not multiples of 8 (an RGB stem: C = 3) or
 * whose tensors are not 16-byte aligned: x (NHWC) is copied to C rounded up to 8 channels, the
 * weights ([R][S][C][K]) to C and K rounded up, the convolution runs on the padded tensors
 * (zero channels add exact zeros) and the K valid channels of every output pixel are copied to
 * y (NPQK, dense).  Geometry, dilation and ep as for alcop_conv2d_igemm_dilated; sched: a
 * schedule for the padded problem or NULL.  workspace: at least
 * alcop_conv2d_unaligned_workspace_bytes(...) bytes, otherwise as above.
 */
size_t alcop_conv2d_unaligned_workspace_bytes(int N, int H, int W, int C, int K, int R, int S,
                                              int stride_h, int stride_w, int pad_h, int pad_w,
                                              int dil_h, int dil_w, alcop_dtype out);
int alcop_conv2d_igemm_unaligned(const void* x, const void* w, void* y, int N, int H, int W, int C,
                                 int K, int R, int S, int stride_h, int stride_w, int pad_h,
                                 int pad_w, int dil_h, int dil_w, alcop_dtype in, alcop_dtype out,
                                 const alcop_epilogue* ep /* host, may be NULL */,
                                 const alcop_sched* sched /* host */, void* workspace,
                                 size_t workspace_bytes, void* hip_stream);

/*
 * Split-K: the reduction axis is cut into `split` slices of whole k-tiles, every slice is a block
 * of its own (grid.z), and a second kernel adds the slices' fp32 partial tiles in ascending
 * order, applies f(.) and converts to the output type.  For outputs with few tiles and a long
 * reduction axis, the case the paper singles out as gaining most from pipelining (Sec. 6.2, the
 * 1024 x 64 output with K = 2048) and where tiling alone leaves most compute units idle
 * (Sec. 1, Fig. 1: tile size against inter-tile parallelism).  The result is deterministic but,
 * unlike every unsplit schedule of a tile, not bit-identical to the unsplit one.
 *   workspace: DEVICE memory, 16-byte aligned, at least alcop_splitk_workspace_bytes(batch, M, N,
 *     split) bytes (4 * split * batch * M * N); owned by the caller, overwritten by the call,
 *     holds nothing afterwards.  Calls that share a workspace must be ordered on one stream.
 *   split: 1..64 slices (fewer are used if K has fewer k-tiles; 1 runs the unsplit kernel's
 *     loop through the workspace), or 0 = the model's choice.
 *   sched: one of the split-K variants built into the library (alcop_splitk_auto returns the
 *     model's pick), or NULL / zero = that pick.  l2_prefetch must be 0.
 *   batch = 1 with strides 0 is a plain GEMM.  Layouts as for alcop_gemm (variants are built for
 *     A stored K x M only together with B stored K x N: the weight-gradient product X^T . dY).
 * Errors as for alcop_gemm; ALCOP_ERR_SIZE also if the workspace is too small.
 */
size_t alcop_splitk_workspace_bytes(int batch, int M, int N, int split);

int alcop_gemm_splitk(const void* A, const void* B, void* C, int batch, int M, int N, int K,
                      long lda, long ldb, long ldc, long strideA, long strideB, long strideC,
                      int transA, int transB, alcop_dtype in, alcop_dtype out,
                      const alcop_epilogue* ep /* host, may be NULL */,
                      const alcop_sched* sched /* host */, int split,
                      void* workspace /* device */, size_t workspace_bytes, void* hip_stream);

/*
 * alcop_gemm_splitk for callers that cannot allocate device memory or are not allowed to: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and bit-identical results, but no workspace argument: the fp32 partial tiles go to
 * an array of ALCOP_SPLITK_STATIC_BYTES that lives in the library's own device image (each GPU
 * the library runs on holds it until the process ends).  The call allocates and frees nothing;
 * the first call on a device looks the array's device address up, which may make the runtime
 * load the library's device code, so make one call on each device before capturing a graph.
 *   ALCOP_ERR_SIZE if 4 * slices * batch * M * N exceeds ALCOP_SPLITK_STATIC_BYTES (checked on
 *   the host before anything touches the device); other errors as for alcop_gemm_splitk.
 * Every call on one GPU uses that GPU's array and nothing in it is kept between calls: calls on
 * different streams of one GPU that overlap in time race on it, so order them (one stream, or
 * events).  Nothing needs clearing: every slice writes its whole M x N partial tile before the
 * second kernel, ordered after it on the stream, reads exactly those.
 */
#define ALCOP_SPLITK_STATIC_BYTES (32u << 20)
int alcop_gemm_splitk_static(const void* A, const void* B, void* C, int batch, int M, int N, int K,
                             long lda, long ldb, long ldc, long strideA, long strideB,
                             long strideC, int transA, int transB, alcop_dtype in, alcop_dtype out,
                             const alcop_epilogue* ep /* host, may be NULL */,
                             const alcop_sched* sched /* host */, int split, void* hip_stream);

/* GEMM view of the convolution: M = N*P*Q, N = K, reduction R*S*C; workspace as above. */
int alcop_conv2d_igemm_splitk(const void* x, const void* w, void* y, int N, int H, int W, int C,
                              int K, int R, int S, int stride_h, int stride_w, int pad_h,
                              int pad_w, alcop_dtype in, alcop_dtype out,
                              const alcop_sched* sched /* host */, int split,
                              void* workspace /* device */, size_t workspace_bytes,
                              void* hip_stream);

/*
 * Model-ranked tuning over (split-K variant, number of slices): candidates whose partial tiles
 * do not fit the workspace are pruned, the rest are ranked by the model of alcop_splitk_auto and
 * the first top_k (0 = all) are timed with HIP events, `iters` launches of both kernels each.
 * Operands as for alcop_tune (C and the workspace are overwritten); best / best_split / best_us
 * receive the fastest measured pair; the optional log arrays (host, log_cap entries) the trials
 * in rank order, log_split holding the number of slices actually launched.  Synchronises.
 */
int alcop_tune_splitk(const alcop_problem* prob /* host */, const void* A, const void* B, void* C,
                      long lda, long ldb, long ldc, long strideA, long strideB, long strideC,
                      const int* conv /* host, 11 ints, conv only */, void* workspace /* device */,
                      size_t workspace_bytes, int top_k, int iters, alcop_sched* best /* host */,
                      int* best_split /* host */, double* best_us /* host */,
                      int* trials_run /* host */, int* space_size /* host */,
                      alcop_sched* log_sched /* host */, int* log_split /* host */,
                      double* log_pred_us /* host */, double* log_meas_us /* host */, int log_cap,
                      void* hip_stream);

/* The split-K variants built into the library for the problem's dtype / layout / operator
 * (same conventions as alcop_sched_space). */
int alcop_splitk_space(const alcop_problem* prob /* host */, alcop_sched* out /* host */, int cap);

/*
 * The (schedule, split) the static model ranks first among the split-K variants: the model of
 * Sec. 5 applied to the sliced problem (batch x split blocks, reduction axis of one slice, fp32
 * output) plus the reduction pass.  split = 0 searches the split as well; predicted_us (host,
 * may be NULL) receives the predicted time.  Host only, launches nothing.
 */
int alcop_splitk_auto(const alcop_problem* prob /* host */, int split,
                      alcop_sched* sched_out /* host */, int* split_out /* host */,
                      double* predicted_us /* host */);

/*
 * Feasibility of a schedule for a problem, without launching (the checks the paper's
 * schedule rules and "compile fail" marks stand for, Sec. 3.1 and Fig. 9): a kernel with
 * these parameters is built; the LDS ring fits 160 KB; the outstanding-load count
 * (S-2)*loads_per_stage fits the 6-bit vector-memory counter; fuse_inner implies R=2, S>=2;
 * for conv a kernel with the gather that C and bk call for.  Returns ALCOP_OK or the error a
 * launch would return.
 */
int alcop_sched_supported(const alcop_problem* prob /* host */, const alcop_sched* sched /* host */);

/*
 * The schedule space: every kernel built into the library that matches the problem's
 * dtype / layout / operator (for a convolution: with the gather that the channel count and the
 * kernel's bk call for), whether or not it is feasible for the shape.
 * Writes at most `cap` entries to out (host) and returns the total count, or a negative
 * alcop_status if the problem itself is invalid.
 */
int alcop_sched_space(const alcop_problem* prob /* host */, alcop_sched* out /* host */, int cap);

/*
 * The kernels outside the default space built for the problem.  They run when a caller names
 * them or asks the tuner for them (alcop_tune with variants = 1); a NULL / zero schedule never
 * resolves to one unless the tuner chose it.  They are
 *   - the schedule variant 1, whose feasibility depends on more than the
 *     problem description: for a convolution the variant with the input patch resident in LDS,
 *     which also needs stride 1 and a patch that fits the LDS (alcop_sched_supported only checks
 *     that such a kernel exists; the launch or the tuner checks the rest);
 *   - the kernels with bk = 128: half as many block-wide synchronisations per unit of work, but
 *     two stages of a 128 x 128 tile already fill 128 KB of LDS;
 *   - the persistent kernels whose consumers run the deep register pipeline (variant 2 with
 *     reg_stages = 4): measured no faster than reg_stages = 2 on any shape tried.
 */
int alcop_sched_variants(const alcop_problem* prob /* host */, alcop_sched* out /* host */, int cap);

/*
 * Static latency model (paper Sec. 5, Table 1): predicted kernel time in microseconds and,
 * optionally, its terms.  terms (host, may be NULL) receives 8 doubles:
 *   [0] T_kernel  [1] T_threadblk  [2] T_init  [3] T_main_loop  [4] T_epilogue
 *   [5] T_smem_load  [6] T_smem_use  [7] N_threadblk_batch
 * model: 0 = the paper's pipeline-aware model; 1 = the bottleneck-only model it is compared
 * against in Sec. 6.4 (max of compute, LDS traffic and DRAM traffic at full rate).
 * One deliberate deviation from Table 1: the multiplexing factor of the register-level pipeline
 * is the number of wavefronts per SIMD, not the number of warps per threadblock (a wavefront is
 * pinned to one of a compute unit's four matrix pipes).  A schedule of variant 2 is predicted
 * like the default kernel of the same tile and stage count.
 */
int alcop_model_predict(const alcop_problem* prob /* host */, const alcop_sched* sched /* host */,
                        int model, double* predicted_us /* host */, double* terms /* host */);

/*
 * Model-ranked tuning (paper Sec. 5.3 "Analytical-only": rank all schedules by predicted
 * latency and measure the best-ranked ones).  Runs on the caller's buffers (contents of C
 * are overwritten), synchronises the stream, times each trial with HIP events.
 *   top_k > 0: time the top_k feasible schedules by predicted latency, at most max(2, top_k / 4)
 *   of them from one (tile, wave tile, variant) family (the pipelining variants of one tile are
 *   predicted within a few percent of each other and would otherwise fill the budget); with
 *   top_k >= 8 the last trials of the budget go to the one-stage schedule of the two best-ranked
 *   tile families of the tile-at-a-time kernels, unless the budget holds one already (pipelining slows
 *   some operators down, Sec. 6.2, and a static model cannot be trusted to know which);
 *   top_k == 0: time all feasible schedules (exhaustive / grid search, the 100 % reference of
 *   Sec. 6.4).
 *   model: 0 / 1 as in alcop_model_predict (fixed ranking by that model);
 *          2 = measurement-corrected model (Sec. 5.3 "Analytical + ML"): a regression whose prior
 *              is model 0 and which is refitted after every timed trial; the next trial is the
 *              untried schedule with the lowest corrected prediction;
 *          3 = no model: schedules in table order (the paper's grid search baseline).
 *   variants: 0 = candidates are the default kernels (alcop_sched_space); 1 = also the kernels
 *          outside the default space (alcop_sched_variants), those that this call cannot use
 *          being pruned.
 *   For conv problems pass x as A, w as B, y as C and the geometry in `conv` (host; 11 ints:
 *   N,H,W,C,K,R,S,stride_h,stride_w,pad_h,pad_w), else conv = NULL and lda/ldb/ldc/strides
 *   as for alcop_bmm (batch 1 for GEMM).
 *   Outputs (host): best schedule and its time; number of timed trials; size of the feasible
 *   space; optional log arrays (may be NULL) of capacity log_cap receiving, in rank order,
 *   each timed schedule, its predicted and measured microseconds.
 */
int alcop_tune(const alcop_problem* prob /* host */, const void* A, const void* B, void* C,
               long lda, long ldb, long ldc, long strideA, long strideB, long strideC,
               const int* conv /* host */, int top_k, int model, int variants, int iters,
               alcop_sched* best /* host */, double* best_us /* host */,
               int* trials_run /* host */, int* space_size /* host */,
               alcop_sched* log_sched /* host */, double* log_pred_us /* host */,
               double* log_meas_us /* host */, int log_cap, void* hip_stream);

/*
 * The learner behind alcop_tune(model = 2) on its own, host only (paper Sec. 5.3, "Analytical +
 * ML": a cost model that starts from the analytical predictions and is corrected by profiled
 * trials).  It is a ridge regression on log(microseconds) over ALCOP_CORRECTOR_DIM features of a
 * (problem, schedule) pair whose prior weight vector is (0, 1, 0, ...): with no trials it predicts
 * exactly the analytical model.
 *   alcop_corrector_features writes the features of one pair: 1; log of the prediction of model
 *     0; log of the prediction of model 1; log2(bm * bn) - 14; log2(bk) - 6; stages - 2;
 *     reg_stages - 1; fuse_inner; log2(waves per block) - 2; 1 if l2_prefetch > 0.
 *   alcop_corrector_fit takes n trials (x: n rows of features, row-major; measured_us: n times,
 *     all > 0) and writes the weights w that minimise sum (log t - w.x)^2 + 0.3 |w - prior|^2,
 *     i.e. the solution of (X'X + 0.3 I) w = X' log t + 0.3 prior; n = 0 gives the prior.
 */
#define ALCOP_CORRECTOR_DIM 10
int alcop_corrector_features(const alcop_problem* prob /* host */, const alcop_sched* sched /* host */,
                             double* x /* host, ALCOP_CORRECTOR_DIM */);
int alcop_corrector_fit(const double* x /* host */, const double* measured_us /* host */, int n,
                        double* weights /* host, ALCOP_CORRECTOR_DIM */);

/*
 * The order in which alcop_tune(top_k, model 0 or 1) tries the schedules of a problem (those that
 * only the call's geometry could still prune included): by predicted latency with the per-family
 * cap and the one-stage trials described there.  Host only.  Writes up to cap schedules, returns their total number.
 */
int alcop_sched_ranked(const alcop_problem* prob /* host */, int model, int variants, int top_k,
                       alcop_sched* out /* host */, int cap);

/*
 * The schedule a NULL / zero schedule argument resolves to for this problem: the entry of the
 * tuning cache if there is one (written by alcop_tune or alcop_cache_load), else the feasible
 * schedule with the lowest predicted latency under model 0.  Host only, launches nothing.
 */
int alcop_sched_auto(const alcop_problem* prob /* host */, alcop_sched* out /* host */);

/*
 * Tuning cache on disk (the tuner's trial outcome per problem, so that a later process skips the
 * timing).  Text file, one line per problem:
 *   op batch M N K transA transB in out conv_C : bm bn bk wm wn stages reg_stages fuse raster l2 variant
 * (the last number may be missing in files written before the field existed: 0)
 * alcop_cache_save writes every cached entry and returns their number; alcop_cache_load merges
 * the file's entries into the cache (entries that name a schedule this library cannot run for
 * that problem are skipped) and returns the number accepted.  Negative return = alcop_status.
 * If the environment variable ALCOP_LOG is set (to anything), every launch prints one line to
 * stderr: the problem, the schedule it resolved to, the grid and the LDS size.
 * If the environment variable ALCOP_TUNE_CACHE names a file, it is merged in once, before the
 * first time a NULL / zero schedule is resolved (a missing or unreadable file is ignored).
 */
int alcop_cache_save(const char* path /* host */);
int alcop_cache_load(const char* path /* host */);

/* Times `iters` back-to-back launches of one schedule with HIP events on the given stream
 * (after `warmup` untimed ones); writes the mean microseconds per launch.  Same operand
 * conventions as alcop_tune.  Synchronises the stream. */
int alcop_time(const alcop_problem* prob /* host */, const void* A, const void* B, void* C,
               long lda, long ldb, long ldc, long strideA, long strideB, long strideC,
               const int* conv /* host */, const alcop_sched* sched /* host */,
               int warmup, int iters, double* mean_us /* host */, void* hip_stream);

/* Static string for a status code. */
/*
 * Optional: does now, on the current device, what the first call of each entry point would do
 * besides launching (opting every kernel in to its LDS size, looking up the device array of
 * alcop_gemm_splitk_static, reading the compute-unit count).  After it, a first call is as cheap
 * as any other and may be recorded into a HIP graph without an eager call before the capture.
 * Launches nothing, allocates nothing.  Returns ALCOP_OK or ALCOP_ERR_LAUNCH (no usable device).
 */
int alcop_init(void);

const char* alcop_strerror(int code);

/* Library version, and the GPU architecture string it was compiled for ("gfx950"). */
const char* alcop_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ALCOP_H */
