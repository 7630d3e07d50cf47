/*
 * CPU oracle for the operators: GEMM, batched matmul, 2-D convolution, GEMV and 2-D
 * average pooling.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the GPU
 * kernels must compute; it shares no code with them.  Only tests, the smoke check and
 * the cpu_baseline leg of the benchmark may call it.
 *
 * Every operator is the textbook definition written out as nested loops:
 *   GEMM   C_ij = alpha * sum_k A_ik B_kj + beta * C_ij        (operator table, GEMM row)
 *   BMM    the same for every batch index, with element strides between batches
 *   Conv2d O = (I * K) downsampled by S on NCHW input and KCRS filters, read as a
 *          cross-correlation (no filter flip) with explicit symmetric zero padding
 *          (operator table, Conv2d row)
 *   GEMV   y_i = alpha * sum_n A_in x_n + beta * y_i             (operator table, GEMV row)
 *   AvgPooling2d  O_xy = (1/F^2) sum_ij I_{S x + i, S y + j}      (operator table, AvgPooling2d row)
 * Inputs are decoded from their stored bits (fp32, IEEE half, bfloat16) to double
 * exactly; products and sums are carried in double, in index order.  There is no
 * blocking, no reordering and no library call.  OpenMP only splits the outermost
 * output loop across host threads; each output element is still one serial sum.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2 };

/* IEEE 754 binary16 -> double, exact: sign(1) exponent(5, bias 15) fraction(10). */
static double half_bits_to_double(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int expo = (b >> 10) & 0x1F;
    int frac = b & 0x3FF;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);                /* zero and subnormals: frac * 2^-24 */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp((double)(frac + 1024), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    return sign ? -v : v;
}

/* bfloat16 is the upper half of an IEEE binary32. */
static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

double oracle_decode(int dtype, const void *base, int64_t idx)
{
    switch (dtype) {
    case ORACLE_F32:  return (double)((const float *)base)[idx];
    case ORACLE_F16:  return half_bits_to_double(((const uint16_t *)base)[idx]);
    case ORACLE_BF16: return bf16_bits_to_double(((const uint16_t *)base)[idx]);
    default:          return NAN;
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Element (i,k) of op(A), where A is stored [M][K] (transA=0) or [K][M] (transA=1). */
static double a_at(int dtype, const void *A, int64_t lda, int transA, int64_t i, int64_t k)
{
    return oracle_decode(dtype, A, transA ? k * lda + i : i * lda + k);
}

/* Element (k,j) of op(B), where B is stored [K][N] (transB=0) or [N][K] (transB=1). */
static double b_at(int dtype, const void *B, int64_t ldb, int transB, int64_t k, int64_t j)
{
    return oracle_decode(dtype, B, transB ? j * ldb + k : k * ldb + j);
}

static double gemm_entry(int dtype, int transA, int transB, int64_t K,
                         const void *A, int64_t lda, const void *B, int64_t ldb,
                         int64_t i, int64_t j)
{
    double acc = 0.0;
    for (int64_t k = 0; k < K; ++k)
        acc += a_at(dtype, A, lda, transA, i, k) * b_at(dtype, B, ldb, transB, k, j);
    return acc;
}

/*
 * C (double, row-major, leading dimension ldc) <- alpha * op(A) op(B) + beta * C.
 * beta == 0 does not read C.
 */
int oracle_gemm(int dtype, int transA, int transB, int64_t M, int64_t N, int64_t K,
                double alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                double beta, double *C, int64_t ldc)
{
    if (dtype < 0 || dtype > 2 || M < 0 || N < 0 || K < 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double s = alpha * gemm_entry(dtype, transA, transB, K, A, lda, B, ldb, i, j);
            if (beta != 0.0) s += beta * C[i * ldc + j];
            C[i * ldc + j] = s;
        }
    return 0;
}

/* Byte size of one stored element. */
static int64_t esize(int dtype) { return dtype == ORACLE_F32 ? 4 : 2; }

int oracle_bmm(int dtype, int transA, int transB, int64_t batch, int64_t M, int64_t N, int64_t K,
               double alpha, const void *A, int64_t lda, int64_t strideA,
               const void *B, int64_t ldb, int64_t strideB,
               double beta, double *C, int64_t ldc, int64_t strideC)
{
    if (dtype < 0 || dtype > 2 || batch < 0) return 1;
    for (int64_t b = 0; b < batch; ++b) {
        const char *Ab = (const char *)A + b * strideA * esize(dtype);
        const char *Bb = (const char *)B + b * strideB * esize(dtype);
        int rc = oracle_gemm(dtype, transA, transB, M, N, K, alpha, Ab, lda, Bb, ldb,
                             beta, C + b * strideC, ldc);
        if (rc) return rc;
    }
    return 0;
}

/* alpha * sum only, at `count` chosen coordinates (b, i, j); for full-size spot checks. */
int oracle_bmm_at(int dtype, int transA, int transB, int64_t K, double alpha,
                  const void *A, int64_t lda, int64_t strideA,
                  const void *B, int64_t ldb, int64_t strideB,
                  int64_t count, const int64_t *bij, double *out)
{
    if (dtype < 0 || dtype > 2) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < count; ++t) {
        int64_t b = bij[3 * t], i = bij[3 * t + 1], j = bij[3 * t + 2];
        const char *Ab = (const char *)A + b * strideA * esize(dtype);
        const char *Bb = (const char *)B + b * strideB * esize(dtype);
        out[t] = alpha * gemm_entry(dtype, transA, transB, K, Ab, lda, Bb, ldb, i, j);
    }
    return 0;
}

static int64_t conv_out_extent(int64_t in, int64_t filt, int64_t stride, int64_t pad)
{
    int64_t span = in + 2 * pad - filt;
    return span < 0 ? 0 : span / stride + 1;
}

static double conv_entry(int dtype, int64_t C, int64_t H, int64_t W, int64_t R, int64_t S,
                         int64_t stride, int64_t pad, const void *I, const void *Wt,
                         int64_t n, int64_t k, int64_t p, int64_t q)
{
    double acc = 0.0;
    for (int64_t c = 0; c < C; ++c)
        for (int64_t r = 0; r < R; ++r)
            for (int64_t s = 0; s < S; ++s) {
                int64_t y = p * stride - pad + r;
                int64_t x = q * stride - pad + s;
                if (y < 0 || y >= H || x < 0 || x >= W) continue;   /* zero padding */
                double in = oracle_decode(dtype, I, ((n * C + c) * H + y) * W + x);
                double wt = oracle_decode(dtype, Wt, ((k * C + c) * R + r) * S + s);
                acc += in * wt;
            }
    return acc;
}

/*
 * O[n][k][p][q] (double, contiguous) = sum_{c,r,s} I[n][c][p*stride-pad+r][q*stride-pad+s] * W[k][c][r][s]
 * with P = floor((H + 2 pad - R)/stride) + 1, Q likewise.
 */
int oracle_conv2d(int dtype, int64_t N, int64_t C, int64_t H, int64_t W,
                  int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad,
                  const void *I, const void *Wt, double *O)
{
    if (dtype < 0 || dtype > 2 || stride < 1 || pad < 0) return 1;
    int64_t P = conv_out_extent(H, R, stride, pad), Q = conv_out_extent(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            for (int64_t p = 0; p < P; ++p)
                for (int64_t q = 0; q < Q; ++q)
                    O[((n * K + k) * P + p) * Q + q] =
                        conv_entry(dtype, C, H, W, R, S, stride, pad, I, Wt, n, k, p, q);
    return 0;
}

int oracle_conv2d_at(int dtype, int64_t N, int64_t C, int64_t H, int64_t W,
                     int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad,
                     const void *I, const void *Wt,
                     int64_t count, const int64_t *nkpq, double *out)
{
    (void)N; (void)K;
    if (dtype < 0 || dtype > 2 || stride < 1 || pad < 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < count; ++t)
        out[t] = conv_entry(dtype, C, H, W, R, S, stride, pad, I, Wt,
                            nkpq[4 * t], nkpq[4 * t + 1], nkpq[4 * t + 2], nkpq[4 * t + 3]);
    return 0;
}

/*
 * GEMV: y_i = alpha * sum_n A_in x_n + beta * y_i, i in [0, M)   (operator table, GEMV row).
 * A is row-major with leading dimension lda; one serial double sum per output, in index
 * order.  y holds the prior values on entry (read only if beta != 0) and the result on exit.
 */
int oracle_gemv(int dtype, int64_t M, int64_t N, double alpha, const void *A, int64_t lda,
                const void *x, double beta, double *y)
{
    if (dtype < 0 || dtype > 2 || M < 0 || N < 0 || lda < N) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double acc = 0.0;
        for (int64_t n = 0; n < N; ++n)
            acc += oracle_decode(dtype, A, i * lda + n) * oracle_decode(dtype, x, n);
        y[i] = alpha * acc + (beta != 0.0 ? beta * y[i] : 0.0);
    }
    return 0;
}

/*
 * AvgPooling2d: O[n][c][x][y] = (1/F^2) * sum_{i<F} sum_{j<F} I[n][c][S*x + i][S*y + j]
 * (operator table, AvgPooling2d row) on an NCHW input, no padding; the output extent is
 * floor((H - F)/S) + 1 by floor((W - F)/S) + 1 (windows that would leave the image do not
 * exist).  The window is summed in double in (i, j) order, then divided once by F*F.
 */
static double pool_entry(int dtype, int64_t H, int64_t W, int64_t F, int64_t S, const void *I,
                         int64_t plane, int64_t p, int64_t q)
{
    double acc = 0.0;
    for (int64_t i = 0; i < F; ++i)
        for (int64_t j = 0; j < F; ++j)
            acc += oracle_decode(dtype, I, (plane * H + S * p + i) * W + S * q + j);
    return acc / (double)(F * F);
}

int oracle_avgpool2d(int dtype, int64_t N, int64_t C, int64_t H, int64_t W, int64_t F, int64_t S,
                     const void *I, double *O)
{
    if (dtype < 0 || dtype > 2 || F < 1 || S < 1 || H < F || W < F) return 1;
    int64_t P = (H - F) / S + 1, Q = (W - F) / S + 1;
#pragma omp parallel for schedule(static)
    for (int64_t plane = 0; plane < N * C; ++plane)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q)
                O[(plane * P + p) * Q + q] = pool_entry(dtype, H, W, F, S, I, plane, p, q);
    return 0;
}

/* The same for `count` output coordinates (n, c, p, q) given as a flat int64 array. */
int oracle_avgpool2d_at(int dtype, int64_t C, int64_t H, int64_t W, int64_t F, int64_t S,
                        const void *I, int64_t count, const int64_t *ncpq, double *out)
{
    if (dtype < 0 || dtype > 2 || F < 1 || S < 1 || H < F || W < F) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < count; ++t)
        out[t] = pool_entry(dtype, H, W, F, S, I, ncpq[4 * t] * C + ncpq[4 * t + 1], ncpq[4 * t + 2], ncpq[4 * t + 3]);
    return 0;
}
