/*
 * CPU oracle for the ALCOP hot path: GEMM, batched matmul and 2-D convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product library links, loads or
 * imports this file; only tests, the smoke check and the cpu_baseline leg of the
 * benchmark use it.  It shares no code with the GPU path.
 *
 * What it computes.  Load-compute pipelining is a transformation of a
 * load-and-use loop that leaves the computed values unchanged (paper Sec. 3,
 * opening paragraphs, and Sec. 4): the pipelined kernels reach exactly the
 * plain definition of the operator.  The operators are the three the paper
 * names as pipelinable (Sec. 6.2: MatMul, BMM, Conv2D), with half-precision
 * inputs (Sec. 6.1).  The oracle is therefore the definition written out:
 *
 *   GEMM    C[i][j]       = sum_{k=0..K-1} A(i,k) * B(k,j)
 *   BMM     C[b][i][j]    = the same for every batch index b
 *   Conv2D  y[n][p][q][k] = sum_{r,s,c} x[n][p*sh-ph+r][q*sw-pw+s][c] * w[r][s][c][k]
 *           (cross-correlation, zero outside the image, NHWC input,
 *            RSCK weights, NPQK output)
 *
 * Inputs are the 16-bit patterns (IEEE binary16 or bfloat16) that the GPU also
 * receives.  They are decoded exactly to double; every sum runs in double with
 * the reduction index ascending (k, or (r,s,c) lexicographic for the
 * convolution).  No blocking, no fusion, no reordering of the reduction.
 *
 * Pins (tests/test_oracle_*.py): both decoders against every one of the 65536
 * patterns as converted by numpy / torch; brute-force pure-Python loops on
 * tiny shapes; identity and permutation operands; all-ones and rank-1 closed
 * forms; exact int64 arithmetic on small-integer inputs; im2col + GEMM as a
 * second route for the convolution; centre/off-centre delta taps; tap counts
 * at the image border.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1 };

/* IEEE 754 binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
double alcop_oracle_decode_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);               /* subnormal: m * 2^-10 * 2^-14 */
    else if (e == 31)
        v = m ? (double)NAN : (double)INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);   /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* bfloat16: 1 sign, 8 exponent (bias 127), 7 fraction bits. */
double alcop_oracle_decode_bf16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 7) & 0xff;
    int m = h & 0x7f;
    double v;
    if (e == 0)
        v = ldexp((double)m, -133);              /* subnormal: m * 2^-7 * 2^-126 */
    else if (e == 255)
        v = m ? (double)NAN : (double)INFINITY;
    else
        v = ldexp((double)(m + 128), e - 134);   /* (1 + m/128) * 2^(e-127) */
    return sign ? -v : v;
}

static double decode(uint16_t h, int dtype)
{
    return dtype == ORACLE_BF16 ? alcop_oracle_decode_bf16(h) : alcop_oracle_decode_f16(h);
}

void alcop_oracle_decode(const uint16_t *bits, double *out, size_t n, int dtype)
{
    for (size_t i = 0; i < n; i++)
        out[i] = decode(bits[i], dtype);
}

int alcop_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * C (double, row-major, leading dimension ldc) = A * B.
 * transA == 0: A(i,k) = A[i*lda + k]   (M x K row-major)
 * transA == 1: A(i,k) = A[k*lda + i]   (stored K x M)
 * transB == 0: B(k,j) = B[k*ldb + j]   (K x N row-major)
 * transB == 1: B(k,j) = B[j*ldb + k]   (stored N x K, the Q.K^T case)
 * Loop order i, k, j: each C[i][j] still receives its K terms with k ascending.
 * Returns 0, or -1 if memory for the decoded copy of B cannot be obtained.
 */
int alcop_oracle_gemm(const uint16_t *A, const uint16_t *B, double *C,
                      int M, int N, int K, long lda, long ldb, long ldc,
                      int transA, int transB, int dtype)
{
    double *Bd = (double *)malloc((size_t)K * (size_t)N * sizeof(double) + 8);
    if (!Bd)
        return -1;
    for (int k = 0; k < K; k++)
        for (int j = 0; j < N; j++) {
            uint16_t b = transB ? B[(size_t)j * ldb + k] : B[(size_t)k * ldb + j];
            Bd[(size_t)k * N + j] = decode(b, dtype);
        }
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; i++) {
        double *c = C + (size_t)i * ldc;
        for (int j = 0; j < N; j++)
            c[j] = 0.0;
        for (int k = 0; k < K; k++) {
            uint16_t ab = transA ? A[(size_t)k * lda + i] : A[(size_t)i * lda + k];
            double a = decode(ab, dtype);
            const double *b = Bd + (size_t)k * N;
            for (int j = 0; j < N; j++)
                c[j] += a * b[j];
        }
    }
    free(Bd);
    return 0;
}

/* Batched: operand b starts at base + b*stride (strides in elements). */
int alcop_oracle_bmm(const uint16_t *A, const uint16_t *B, double *C, int batch,
                     int M, int N, int K, long lda, long ldb, long ldc,
                     long strideA, long strideB, long strideC,
                     int transA, int transB, int dtype)
{
    for (int b = 0; b < batch; b++) {
        int rc = alcop_oracle_gemm(A + (size_t)b * strideA, B + (size_t)b * strideB,
                                   C + (size_t)b * strideC, M, N, K, lda, ldb, ldc,
                                   transA, transB, dtype);
        if (rc)
            return rc;
    }
    return 0;
}

/*
 * Direct convolution, seven loops.
 * x: [N][H][W][C], w: [R][S][C][K], y (double): [N][P][Q][K],
 * P = (H + 2*pad_h - R)/stride_h + 1, Q likewise.
 */
int alcop_oracle_conv2d(const uint16_t *x, const uint16_t *w, double *y,
                        int N, int H, int W, int C, int K, int R, int S,
                        int stride_h, int stride_w, int pad_h, int pad_w, int dtype)
{
    int P = (H + 2 * pad_h - R) / stride_h + 1;
    int Q = (W + 2 * pad_w - S) / stride_w + 1;
    size_t wn = (size_t)R * S * C * K;
    double *wd = (double *)malloc(wn * sizeof(double) + 8);
    if (!wd)
        return -1;
    for (size_t i = 0; i < wn; i++)
        wd[i] = decode(w[i], dtype);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; n++)
        for (int p = 0; p < P; p++)
            for (int q = 0; q < Q; q++) {
                double *out = y + (((size_t)n * P + p) * Q + q) * K;
                for (int k = 0; k < K; k++)
                    out[k] = 0.0;
                for (int r = 0; r < R; r++) {
                    int ih = p * stride_h - pad_h + r;
                    if (ih < 0 || ih >= H)
                        continue;
                    for (int s = 0; s < S; s++) {
                        int iw = q * stride_w - pad_w + s;
                        if (iw < 0 || iw >= W)
                            continue;
                        const uint16_t *xp = x + (((size_t)n * H + ih) * W + iw) * C;
                        for (int c = 0; c < C; c++) {
                            double xv = decode(xp[c], dtype);
                            const double *wp = wd + (((size_t)r * S + s) * C + c) * K;
                            for (int k = 0; k < K; k++)
                                out[k] += xv * wp[k];
                        }
                    }
                }
            }
    free(wd);
    return 0;
}

/*
 * Dilated convolution (an extension for real workloads; the paper's operators have dilation 1):
 * tap (r, s) reads x[n][p*stride_h - pad_h + r*dil_h][q*stride_w - pad_w + s*dil_w][c], zero
 * outside the image; P = (H + 2*pad_h - dil_h*(R-1) - 1)/stride_h + 1, Q likewise.  Same seven
 * loops and the same summation order (r, s, c ascending) as alcop_oracle_conv2d.
 */
int alcop_oracle_conv2d_dilated(const uint16_t *x, const uint16_t *w, double *y,
                                int N, int H, int W, int C, int K, int R, int S,
                                int stride_h, int stride_w, int pad_h, int pad_w,
                                int dil_h, int dil_w, int dtype)
{
    int P = (H + 2 * pad_h - dil_h * (R - 1) - 1) / stride_h + 1;
    int Q = (W + 2 * pad_w - dil_w * (S - 1) - 1) / stride_w + 1;
    size_t wn = (size_t)R * S * C * K;
    double *wd = (double *)malloc(wn * sizeof(double) + 8);
    if (!wd)
        return -1;
    for (size_t i = 0; i < wn; i++)
        wd[i] = decode(w[i], dtype);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; n++)
        for (int p = 0; p < P; p++)
            for (int q = 0; q < Q; q++) {
                double *out = y + (((size_t)n * P + p) * Q + q) * K;
                for (int k = 0; k < K; k++)
                    out[k] = 0.0;
                for (int r = 0; r < R; r++) {
                    int ih = p * stride_h - pad_h + r * dil_h;
                    if (ih < 0 || ih >= H)
                        continue;
                    for (int s = 0; s < S; s++) {
                        int iw = q * stride_w - pad_w + s * dil_w;
                        if (iw < 0 || iw >= W)
                            continue;
                        const uint16_t *xp = x + (((size_t)n * H + ih) * W + iw) * C;
                        for (int c = 0; c < C; c++) {
                            double xv = decode(xp[c], dtype);
                            const double *wp = wd + (((size_t)r * S + s) * C + c) * K;
                            for (int k = 0; k < K; k++)
                                out[k] += xv * wp[k];
                        }
                    }
                }
            }
    free(wd);
    return 0;
}
