/*
 * CPU oracle for the operator hot path: row softmax, LayerNorm, (batched) GEMM and
 * 2-D convolution, and for the streaming operators added next to them (RMS norm, mean
 * along an axis, add / mul / relu), written out as their plain definitions in double
 * precision.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  It shares no code with the HIP
 * kernels.  The paper defines its operators as compositions of element-wise,
 * broadcast, reduction and expression-as-location operations (Table "Supported
 * representation features", Section 2.1) over dense tensors of the shapes in the
 * table "ML operators optimized using PerfLLM" (Section 4.3); the formulas themselves
 * are the standard (ONNX) ones, which is the operator set the paper says its
 * representation covers (Section 2.1).
 *
 * Every function takes inputs already widened (exactly) to double and writes double
 * results; oracle_round_* round a double result ONCE to the output type.
 * No blocking, no fusion, no reordering: loops run in index order.  OpenMP is used
 * only across independent outputs (rows, output rows), never inside a reduction.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Row softmax (Fig. "Softmax kernel representations", Section 2.1; standard definition):
 *   t_ij = s * x_ij ;  m_i = max_j t_ij ;  e_ij = exp(t_ij - m_i) ;  z_i = sum_j e_ij ;
 *   y_ij = e_ij / z_i.
 * x: rows x cols, row stride ldx; y: row stride ldy. */
void oracle_softmax(const double *x, double *y, int64_t rows, int64_t cols,
                    int64_t ldx, int64_t ldy, double scale)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        const double *xi = x + i * ldx;
        double *yi = y + i * ldy;
        double m = scale * xi[0];
        for (int64_t j = 1; j < cols; ++j) {
            double t = scale * xi[j];
            if (t > m) m = t;
        }
        double z = 0.0;
        for (int64_t j = 0; j < cols; ++j) {
            yi[j] = exp(scale * xi[j] - m);
            z += yi[j];
        }
        for (int64_t j = 0; j < cols; ++j) yi[j] = yi[j] / z;
    }
}

/* LayerNorm over the last dimension (table "ML operators ...", Section 4.3; standard
 * definition with the biased 1/D variance and eps inside the square root):
 *   mu = (1/D) sum_j x_j ; var = (1/D) sum_j (x_j - mu)^2 ; r = 1/sqrt(var + eps) ;
 *   y_j = (x_j - mu) * r * gamma_j + beta_j.
 * mean_out / rstd_out (length rows) may be NULL. */
void oracle_layernorm(const double *x, const double *gamma, const double *beta, double *y,
                      double *mean_out, double *rstd_out, int64_t rows, int64_t cols,
                      int64_t ldx, int64_t ldy, double eps)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        const double *xi = x + i * ldx;
        double *yi = y + i * ldy;
        double s = 0.0;
        for (int64_t j = 0; j < cols; ++j) s += xi[j];
        double mu = s / (double)cols;
        double q = 0.0;
        for (int64_t j = 0; j < cols; ++j) {
            double d = xi[j] - mu;
            q += d * d;
        }
        double var = q / (double)cols;
        double r = 1.0 / sqrt(var + eps);
        for (int64_t j = 0; j < cols; ++j) yi[j] = (xi[j] - mu) * r * gamma[j] + beta[j];
        if (mean_out) mean_out[i] = mu;
        if (rstd_out) rstd_out[i] = r;
    }
}

/* (Batched) GEMM: C_b[m][n] = alpha * sum_{k=0}^{K-1} A_b[m][k] * B_b[k][n], summed in
 * index order.  a_col / b_col = 0: row-major (A[m*lda+k], B[k*ldb+n]);
 * = 1: column-major (A[k*lda+m], B[n*ldb+k]).  C is row-major with row stride ldc.
 * Batch b starts at A + b*strideA, B + b*strideB, C + b*strideC. */
void oracle_gemm(const double *A, const double *B, double *C, int64_t M, int64_t N, int64_t K,
                 int a_col, int64_t lda, int b_col, int64_t ldb, int64_t ldc,
                 int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC, double alpha)
{
    const int64_t a_m = a_col ? 1 : lda, a_k = a_col ? lda : 1;
    const int64_t b_k = b_col ? 1 : ldb, b_n = b_col ? ldb : 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < batch; ++b) {
        for (int64_t m = 0; m < M; ++m) {
            const double *Ab = A + b * strideA + m * a_m;
            const double *Bb = B + b * strideB;
            double *Cb = C + b * strideC + m * ldc;
            for (int64_t n = 0; n < N; ++n) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k) acc += Ab[k * a_k] * Bb[k * b_k + n * b_n];
                Cb[n] = alpha * acc;
            }
        }
    }
}

/* sum_k |A[m][k]| * |B[k][n]| with the same indexing as oracle_gemm (no alpha, no batch):
 * the normaliser of the summation-order-independent rounding bound used by the tests. */
void oracle_gemm_absdot(const double *A, const double *B, double *S, int64_t M, int64_t N, int64_t K,
                        int a_col, int64_t lda, int b_col, int64_t ldb, int64_t lds)
{
    const int64_t a_m = a_col ? 1 : lda, a_k = a_col ? lda : 1;
    const int64_t b_k = b_col ? 1 : ldb, b_n = b_col ? ldb : 1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += fabs(A[m * a_m + k * a_k]) * fabs(B[k * b_k + n * b_n]);
            S[m * lds + n] = acc;
        }
}

/* 2-D convolution in the cross-correlation sense (no filter flip), zero padding:
 *   y[n][p][q][k] = sum_{r,s,c} x[n][p*sh - ph + r][q*sw - pw + s][c] * w[k][r][s][c],
 * taps outside [0,H) x [0,W) contribute 0.  x is NHWC, w is KRSC, y is NPQK with
 * P = (H + 2*ph - R)/sh + 1 and Q = (W + 2*pw - S)/sw + 1 (integer division).
 * If absdot is non-NULL it receives sum |x||w| over the same taps. */
void oracle_conv2d(const double *x, const double *w, double *y, double *absdot,
                   int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                   int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    const int64_t P = (H + 2 * ph - R) / sh + 1;
    const int64_t Q = (W + 2 * pw - S) / sw + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q)
                for (int64_t k = 0; k < K; ++k) {
                    double acc = 0.0, aacc = 0.0;
                    for (int64_t r = 0; r < R; ++r) {
                        int64_t ih = p * sh - ph + r;
                        if (ih < 0 || ih >= H) continue;
                        for (int64_t s = 0; s < S; ++s) {
                            int64_t iw = q * sw - pw + s;
                            if (iw < 0 || iw >= W) continue;
                            const double *xp = x + ((n * H + ih) * W + iw) * C;
                            const double *wp = w + ((k * R + r) * S + s) * C;
                            for (int64_t c = 0; c < C; ++c) {
                                acc += xp[c] * wp[c];
                                aacc += fabs(xp[c]) * fabs(wp[c]);
                            }
                        }
                    }
                    y[((n * P + p) * Q + q) * K + k] = acc;
                    if (absdot) absdot[((n * P + p) * Q + q) * K + k] = aacc;
                }
}

/* RMS normalisation over the last dimension ("rmsnorm" row of the operator table, Section
 * 4.3; standard definition):  r_i = 1/sqrt(mean_j x_ij^2 + eps),  y_ij = x_ij * r_i * gamma_j.
 * rrms (nullable) receives r_i. */
void oracle_rmsnorm(const double *x, const double *gamma, double *y, double *rrms, int64_t rows, int64_t cols,
                    double eps)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        const double *xr = x + i * cols;
        double ss = 0.0;
        for (int64_t j = 0; j < cols; ++j) ss += xr[j] * xr[j];
        const double r = 1.0 / sqrt(ss / (double)cols + eps);
        for (int64_t j = 0; j < cols; ++j) y[i * cols + j] = xr[j] * r * gamma[j];
        if (rrms) rrms[i] = r;
    }
}

/* Batch normalisation with batch statistics ("batchnorm" rows of the operator table, Section
 * 4.3; the paper's case study computes the statistics first and then streams, Section 4.3):
 * x is [N][C][HW]; per channel c over all n and positions: mu_c = mean, var_c = biased variance,
 * r_c = 1/sqrt(var_c + eps), y = (x - mu_c) * r_c * gamma_c + beta_c.  mean / rstd (nullable)
 * receive mu_c and r_c.  Two passes per channel, in index order. */
void oracle_batchnorm(const double *x, const double *gamma, const double *beta, double *y, double *mean,
                      double *rstd, int64_t N, int64_t C, int64_t HW, double eps)
{
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < C; ++c) {
        double s = 0.0;
        for (int64_t n = 0; n < N; ++n)
            for (int64_t i = 0; i < HW; ++i) s += x[(n * C + c) * HW + i];
        const double mu = s / (double)(N * HW);
        double q = 0.0;
        for (int64_t n = 0; n < N; ++n)
            for (int64_t i = 0; i < HW; ++i) {
                const double d = x[(n * C + c) * HW + i] - mu;
                q += d * d;
            }
        const double r = 1.0 / sqrt(q / (double)(N * HW) + eps);
        for (int64_t n = 0; n < N; ++n)
            for (int64_t i = 0; i < HW; ++i) {
                const int64_t o = (n * C + c) * HW + i;
                y[o] = (x[o] - mu) * r * gamma[c] + beta[c];
            }
        if (mean) mean[c] = mu;
        if (rstd) rstd[c] = r;
    }
}

/* Mean along one axis of a rows x cols matrix ("reducemean" row of the operator table):
 * axis 1: y_i = (1/cols) sum_j x_ij (length rows); axis 0: y_j = (1/rows) sum_i x_ij (length cols). */
void oracle_reduce_mean(const double *x, double *y, int64_t rows, int64_t cols, int axis)
{
    if (axis == 1) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < rows; ++i) {
            double s = 0.0;
            for (int64_t j = 0; j < cols; ++j) s += x[i * cols + j];
            y[i] = s / (double)cols;
        }
    } else {
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < cols; ++j) {
            double s = 0.0;
            for (int64_t i = 0; i < rows; ++i) s += x[i * cols + j];
            y[j] = s / (double)rows;
        }
    }
}

/* Element-wise operators of the table ("add", "mul", "relu"): op 0: a+b, 1: a*b, 2: max(a,0). */
void oracle_eltwise(int op, const double *a, const double *b, double *y, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) y[i] = op == 0 ? a[i] + b[i] : op == 1 ? a[i] * b[i] : (a[i] > 0.0 ? a[i] : 0.0);
}

/* One rounding of a double to fp32 (round-to-nearest-even: the C conversion under the
 * default rounding mode). */
void oracle_round_f32(const double *v, float *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = (float)v[i];
}

/* One rounding of a double to bfloat16 (1 sign, 8 exponent, 7 fraction bits),
 * round-to-nearest-even, done directly from the double so there is no double rounding.
 * A bf16 value with binary exponent E (|v| in [2^E, 2^(E+1))) lies on a grid of spacing
 * 2^(E-7); below 2^-126 the grid is the subnormal one, spacing 2^-133.  Finite inputs. */
void oracle_round_bf16(const double *v, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        double a = fabs(v[i]);
        float f;
        if (a == 0.0) {
            f = 0.0f;
        } else {
            int e;
            (void)frexp(a, &e);              /* a = frac * 2^e, frac in [0.5, 1) => E = e-1 */
            int E = e - 1;
            if (E < -126) E = -126;
            double q = ldexp(1.0, E - 7);
            double r = nearbyint(a / q) * q;  /* exact scaling; nearbyint is ties-to-even */
            f = (r > 3.3895313892515355e38) ? INFINITY : (float)r; /* max bf16 */
        }
        uint32_t bits;
        memcpy(&bits, &f, sizeof bits);
        out[i] = (uint16_t)((bits >> 16) | (signbit(v[i]) ? 0x8000u : 0u));
    }
}
