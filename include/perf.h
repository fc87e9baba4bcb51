/*
 * perf.h - C ABI of the MI355X (gfx950) operator library.
 *
 * The operators are the ML-library kernels that the paper's search emits and times
 * (table "ML operators optimized using PerfLLM", Section 4.3): row softmax, LayerNorm,
 * dense / batched GEMM and 2-D convolution.  The paper states them as compositions of
 * element-wise, broadcast, reduction and expression-as-location operations over dense
 * tensors (table "Supported representation features", Section 2.1); the formulas are
 * the standard ones of the same names.
 *
 * Conventions shared by every entry point
 *  - All data pointers are DEVICE pointers (HBM), owned by the caller.  The library
 *    allocates no device memory and keeps no state between calls (the operators that need
 *    scratch memory, perf_batchnorm and perf_reduce_mean_ws, take it from the caller;
 *    perf_batchnorm_static uses a fixed device array instead, see there).
 *  - Calls enqueue work on `stream` (a hipStream_t passed as void*; NULL = the default
 *    stream) and return without synchronising.  Buffers must stay alive and unmodified
 *    until the stream has run the enqueued kernels.
 *  - Every argument check runs on the host before any HIP call; a failed check returns
 *    a PERF_ERR_* code and touches neither the device nor the buffers.
 *  - Leading dimensions and strides are in ELEMENTS of the tensor's dtype.
 *  - bf16 is bfloat16 (1-8-7); conversions to bf16 round to nearest even.  Inputs must
 *    be finite; NaN/Inf behaviour is unspecified.
 *  - Outputs must not overlap inputs, except y == x exactly (same pointer, same ld, same
 *    dtype) for perf_softmax and perf_layernorm.
 *  - Kernels use no atomics: results are bit-identical from run to run.
 *  - The calls may be made from several host threads at once (the only shared host state is a
 *    set of idempotent per-kernel attribute settings behind atomic flags); perf_batchnorm_static
 *    is the exception, see there.
 *  - PERF_ERR_LAUNCH is taken from hipGetLastError() after the launch: an error that one of the
 *    caller's own earlier HIP calls left pending is reported by (and cleared by) the next call
 *    into this library.
 */
#ifndef PERF_H
#define PERF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PERF_OK = 0,
    PERF_ERR_NULL = 1,        /* a required pointer is NULL */
    PERF_ERR_SHAPE = 2,       /* a dimension, leading dimension, stride or padding is out of range */
    PERF_ERR_DTYPE = 3,       /* a dtype enum is out of range */
    PERF_ERR_LAYOUT = 4,      /* a layout enum is out of range */
    PERF_ERR_ALIGN = 5,       /* a pointer is not aligned to its element size */
    PERF_ERR_UNSUPPORTED = 6, /* legal but not implemented combination */
    PERF_ERR_LAUNCH = 7       /* the HIP runtime reported an error at launch */
} perf_status;

typedef enum { PERF_F32 = 0, PERF_BF16 = 1 } perf_dtype;
typedef enum { PERF_ROW_MAJOR = 0, PERF_COL_MAJOR = 1 } perf_layout;
typedef void *perf_stream;

/* Row softmax (Fig. "Softmax kernel representations", Section 2.1; shape row of the
 * operator table, Section 4.3).  For each row i of the rows x cols matrix x:
 *     y[i][j] = exp(scale*(x[i][j] - m_i)) / sum_j exp(scale*(x[i][j] - m_i)),
 * where m_i is the row maximum of scale*x divided by scale (the max for scale >= 0, the
 * min for scale < 0).  Arithmetic is fp32.
 *   x, y     device, rows x cols, row stride ldx / ldy (>= cols); dtype PERF_F32 only
 *   scale    finite
 * Errors: NULL (x or y), SHAPE (rows/cols < 1, ld < cols), DTYPE, ALIGN (pointer not
 * 4-byte aligned), UNSUPPORTED (dtype other than f32), LAUNCH. */
perf_status perf_softmax(const void *x, void *y, int64_t rows, int64_t cols,
                         int64_t ldx, int64_t ldy, perf_dtype x_dt, perf_dtype y_dt,
                         float scale, perf_stream stream);

/* LayerNorm over the last dimension (operator table, Section 4.3).  For each row:
 *     mu = mean_j x[j];  var = mean_j (x[j]-mu)^2  (biased);  r = 1/sqrt(var + eps);
 *     y[j] = (x[j]-mu) * r * gamma[j] + beta[j].
 * Statistics and the affine step are fp32; the result is rounded once to y_dt.
 *   x, y             device, rows x cols, row stride ldx / ldy; dtypes f32 or bf16
 *   gamma, beta      device, length cols, dtype param_dt (f32 or bf16)
 *   mean_out, rstd_out  device fp32[rows] or NULL: receive mu and r
 * Errors: NULL (x, gamma, beta, y), SHAPE (rows/cols < 1, ld < cols, eps < 0 or not
 * finite), DTYPE, ALIGN (pointer not aligned to its element size), LAUNCH. */
perf_status perf_layernorm(const void *x, const void *gamma, const void *beta, void *y,
                           float *mean_out, float *rstd_out, int64_t rows, int64_t cols,
                           int64_t ldx, int64_t ldy, float eps, perf_dtype x_dt,
                           perf_dtype param_dt, perf_dtype y_dt, perf_stream stream);

/* Dense and batched GEMM (operator table rows "matmul" and "bmm", Section 4.3):
 *     C_b[m][n] = alpha * sum_{k<K} A_b[m][k] * B_b[k][n],   b = 0..batch-1,
 * bf16 (or f32) operands, fp32 accumulation, one rounding to c_dt.
 *   A   row-major: A[m*lda + k] (lda >= K);  column-major: A[k*lda + m] (lda >= M)
 *   B   row-major: B[k*ldb + n] (ldb >= N);  column-major: B[n*ldb + k] (ldb >= K)
 *   C   row-major, C[m*ldc + n] (ldc >= N), dtype f32 or bf16
 *   batch >= 1; matrix b starts strideA/strideB/strideC elements after matrix b-1
 *   (strides >= 0; strideC must be >= the extent of one C when batch > 1).
 * The bf16 MFMA path is taken for bf16 operands with A row-major and B column-major (both
 * K-contiguous), K a multiple of 32, lda/ldb/strides multiples of 8 and 16-byte aligned
 * pointers; every other legal combination (fp32 operands, other layouts, any K) runs a kernel
 * built on the fp32 matrix instruction.
 * Errors: NULL, SHAPE, DTYPE, LAYOUT, ALIGN (pointer not aligned to its element size),
 * UNSUPPORTED (f32 operands with bf16 C), LAUNCH. */
perf_status perf_gemm(const void *A, const void *B, void *C, int64_t M, int64_t N, int64_t K,
                      perf_layout la, int64_t lda, perf_layout lb, int64_t ldb, int64_t ldc,
                      int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC,
                      float alpha, perf_dtype ab_dt, perf_dtype c_dt, perf_stream stream);

/* 2-D convolution as an implicit GEMM (operator table rows "conv", Section 4.3;
 * expression-as-location indexing, Section 2.1), cross-correlation with zero padding:
 *     y[n][p][q][k] = sum_{r<R, s<S, c<C} x[n][p*stride_h - pad_h + r][q*stride_w - pad_w + s][c]
 *                                          * w[k][r][s][c],
 * taps outside the image contribute 0;  P = (H + 2*pad_h - R)/stride_h + 1, Q likewise.
 *   x  device, NHWC dense;  w  device, KRSC dense;  y  device, NPQK dense
 *   xw_dt  dtype of x and w (bf16 or f32);  y_dt  f32 or bf16;  fp32 accumulation.
 * The bf16 MFMA path is taken for bf16 x/w with C a multiple of 32 and 16-byte aligned
 * pointers; fp32 x/w (and bf16 with other channel counts) with at least 32 output channels run
 * an implicit GEMM on the fp32 matrix instruction; the remaining cases run direct kernels.
 * Errors: NULL, SHAPE (any dim < 1, stride < 1, pad < 0, filter larger than the padded
 * image, more than 2^31-1 output pixels), DTYPE, ALIGN, LAUNCH. */
perf_status perf_conv2d(const void *x, const void *w, void *y, int64_t N, int64_t H, int64_t W,
                        int64_t C, int64_t K, int64_t R, int64_t S, int64_t stride_h,
                        int64_t stride_w, int64_t pad_h, int64_t pad_w, perf_dtype xw_dt,
                        perf_dtype y_dt, perf_stream stream);

/* Batched score GEMM with the row softmax fused into it (the "bmm" followed by "softmax"
 * pair of the operator table, Section 4.3, joined as the paper's fusion moves join a
 * producer with its consumer, Sections 2.2 and 3.1):
 *     P_b = softmax_rows(alpha * A_b * B_b^T),   b = 0 .. batch-1,
 * i.e. perf_gemm with A row-major (M x K, ld lda) and B column-major (N rows of K, ld ldb)
 * followed by perf_softmax (scale 1) on every row of the M x N result, with the same
 * arithmetic (fp32 accumulation, fp32 softmax) and the same max convention.
 *   A, B     device, bf16 or f32 (ab_dt);  P  device, M x N, row stride ldp, f32 or bf16
 * For bf16 operands with K = 64 or 128, N <= 512 and 16-byte aligned rows the scores never
 * reach memory (one kernel; its exponential is exp2 of a plain fp32 product, relative error
 * about 2^-24 times the exponent); other legal cases run the two operators one
 * after the other through P, which then must be f32 (bf16 P: UNSUPPORTED).
 * Errors: NULL, SHAPE (dimension < 1, ld too small, negative stride, batches overlapping in
 * P, alpha not finite), DTYPE, ALIGN, UNSUPPORTED, LAUNCH. */
perf_status perf_gemm_softmax(const void *A, const void *B, void *P, int64_t M, int64_t N,
                              int64_t K, int64_t lda, int64_t ldb, int64_t ldp, int64_t batch,
                              int64_t strideA, int64_t strideB, int64_t strideP, float alpha,
                              perf_dtype ab_dt, perf_dtype p_dt, perf_stream stream);

/* RMS normalisation over the last dimension ("rmsnorm" row of the operator table, Section
 * 4.3).  For each row:  r = 1/sqrt(mean_j x[j]^2 + eps);  y[j] = x[j] * r * gamma[j].
 * Arithmetic is fp32; the result is rounded once to y_dt.
 *   x, y       device, rows x cols, row stride ldx / ldy; dtypes f32 or bf16
 *   gamma      device, length cols, dtype param_dt;  rrms_out  device fp32[rows] or NULL: receives r
 * y == x exactly is allowed.  Errors as perf_layernorm. */
perf_status perf_rmsnorm(const void *x, const void *gamma, void *y, float *rrms_out, int64_t rows,
                         int64_t cols, int64_t ldx, int64_t ldy, float eps, perf_dtype x_dt,
                         perf_dtype param_dt, perf_dtype y_dt, perf_stream stream);

/* Batch normalisation with batch statistics ("batchnorm" rows of the operator table, Section
 * 4.3; statistics first, then a streaming kernel, as in the paper's case study).  x and y are
 * N x C x H x W, contiguous.  Per channel c, over all n, h, w:
 *     mu = mean x;  var = biased variance;  r = 1/sqrt(var + eps);
 *     y = (x - mu) * r * gamma[c] + beta[c].
 * fp32 statistics (segment statistics merged in double), result rounded once to y_dt.
 *   gamma, beta         device, length C, dtype param_dt
 *   mean_out, rstd_out  device fp32[C] or NULL
 *   workspace           device, at least perf_batchnorm_workspace_bytes(N, C, H, W) bytes, 4-byte
 *                       aligned, owned by the caller; its contents are scratch
 * perf_batchnorm_workspace_bytes returns -1 for a shape perf_batchnorm would reject.
 * y == x exactly is allowed when the dtypes match.
 * Errors: NULL, SHAPE (dimension < 1 or > 2^24, N*C > 65535, eps < 0 or not finite), DTYPE, ALIGN,
 * LAUNCH. */
int64_t perf_batchnorm_workspace_bytes(int64_t N, int64_t C, int64_t H, int64_t W);
perf_status perf_batchnorm(const void *x, const void *gamma, const void *beta, void *y, float *mean_out,
                           float *rstd_out, void *workspace, int64_t N, int64_t C, int64_t H, int64_t W,
                           float eps, perf_dtype x_dt, perf_dtype param_dt, perf_dtype y_dt,
                           perf_stream stream);

/* perf_batchnorm for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operator, same
 * kernels, same results bit for bit; the scratch lives in a file-scope device array of
 * perf_batchnorm_static_max_bytes() (256 KiB) that every GPU the library runs on holds until the
 * process ends.  The call allocates nothing and frees nothing.  Problems whose
 * perf_batchnorm_workspace_bytes exceeds that size return UNSUPPORTED (e.g. 8 x 64 x 300 x 300 needs
 * 37 KiB, 8 x 3 x 2048 x 2048 72 KiB).  All calls on one GPU share the one array: calls that may run
 * concurrently on that GPU (different streams, different host threads) race on it; calls on one
 * stream are safe.  Nothing in the array needs clearing between calls (every word read was
 * written by the same call).
 * Errors: as perf_batchnorm without the workspace checks; LAUNCH also if the array's device
 * address cannot be resolved. */
int64_t perf_batchnorm_static_max_bytes(void);
perf_status perf_batchnorm_static(const void *x, const void *gamma, const void *beta, void *y, float *mean_out,
                                  float *rstd_out, int64_t N, int64_t C, int64_t H, int64_t W, float eps,
                                  perf_dtype x_dt, perf_dtype param_dt, perf_dtype y_dt, perf_stream stream);

/* Mean along one axis of a rows x cols matrix ("reducemean" row of the operator table; the
 * table does not say which axis, both are provided): axis 1: y[i] = mean_j x[i][j] (rows
 * results); axis 0: y[j] = mean_i x[i][j] (cols results).  fp32 accumulation in a fixed order.
 *   x  device, row stride ldx, f32 or bf16;  y  device, contiguous, f32 or bf16
 * Errors: NULL, SHAPE (dimension < 1, ldx < cols, axis not 0 or 1), DTYPE, ALIGN, LAUNCH. */
perf_status perf_reduce_mean(const void *x, void *y, int64_t rows, int64_t cols, int64_t ldx, int axis,
                             perf_dtype x_dt, perf_dtype y_dt, perf_stream stream);

/* The same operator with a caller-supplied workspace.  For axis 0 (16-byte-aligned x, cols and
 * ldx multiples of 16 bytes) the rows are split among workgroups that each sum a 1 KiB-wide
 * column block, and the partial sums are merged in a fixed order by a second kernel: the grid
 * no longer depends on the number of columns and memory is read in long runs.  Every other
 * case is perf_reduce_mean itself.
 *   workspace  device, at least perf_reduce_mean_workspace_bytes(rows, cols, axis, x_dt) bytes,
 *              4-byte aligned, owned by the caller, contents are scratch; may be NULL when
 *              that size is 0 (axis 1, or cols not a multiple of 16 bytes)
 * perf_reduce_mean_workspace_bytes returns -1 for arguments perf_reduce_mean_ws would reject.
 * Errors: as perf_reduce_mean; NULL / ALIGN also for a missing or misaligned workspace. */
int64_t perf_reduce_mean_workspace_bytes(int64_t rows, int64_t cols, int axis, perf_dtype x_dt);
perf_status perf_reduce_mean_ws(const void *x, void *y, void *workspace, int64_t rows, int64_t cols,
                                int64_t ldx, int axis, perf_dtype x_dt, perf_dtype y_dt,
                                perf_stream stream);

/* Element-wise operators of the table ("add", "mul", "relu") on n contiguous elements:
 * y = a + b, a * b, or max(a, 0) (b ignored, may be NULL).  One dtype for all operands;
 * fp32 arithmetic, one rounding to dt.  y may equal a or b exactly.
 * Errors: NULL, SHAPE (n < 0), DTYPE, ALIGN, UNSUPPORTED (op out of range; misaligned buffers
 * of more than 2^26 elements), LAUNCH. */
typedef enum { PERF_ADD = 0, PERF_MUL = 1, PERF_RELU = 2 } perf_eltwise_op;
perf_status perf_eltwise(perf_eltwise_op op, const void *a, const void *b, void *y, int64_t n,
                         perf_dtype dt, perf_stream stream);

/* The same operators with the kernel variant chosen by the caller instead of by the
 * library's shape rules: the knob a timing-driven search turns (the paper's search scores a
 * candidate by the measured runtime of the code it emits, Section 3.2, after validating its
 * output against the untransformed program, Section 3.1; tune.py beside the Python binding
 * does that over these variants).  Arguments, results and errors are those of perf_gemm /
 * perf_conv2d; a variant that cannot run the problem returns UNSUPPORTED.
 *   perf_gemm_variant:  tile = 64, 128 or 256 (workgroup tile edge); kstep = 32 or 64 (main loop;
 *     K must be a multiple of it), or 33 = the K-step-32 loop with its LDS ring deepened to 128 KiB
 *     (16 stages for tile 64, 8 for tile 128, not for 256), or 65 = the K-step-64 loop built on
 *     the 32x32x16 MFMA (tile 256 only, K a multiple of 64); only the bf16 row-major x
 *     column-major case that the MFMA kernels cover has variants.
 *   perf_conv2d_variant: variant 1 = weights in registers (3x3, 64 -> 128 channels, bf16),
 *     2 = implicit GEMM on the shared main loop (bf16, C a multiple of 32), 3 = channel-blocked
 *     direct kernel, 4 = one thread per output, 5 = one filter row per 16-wide MFMA step (bf16,
 *     stride 1, few input channels: 5x5 with 3 channels, 3x3 with 3 or 4; W*C even),
 *     6 = variant 1 with the input rows under a workgroup's pixel range resident in LDS
 *     (stride 1; N*P*Q / 256 pixels per range must divide P*Q, and the rows must fit),
 *     7 = implicit GEMM on the fp32 matrix instruction (any dtype, stride, padding, channel count),
 *     8 = weights in registers with a workgroup per (pixel range, slab of 64 output channels)
 *     and the input rows passing through a ring in LDS (3x3, 64 input channels, bf16, stride 1,
 *     K any multiple of 64, 32 <= Q and a ring of at least 5 rows of 144 Q + 512 bytes within
 *     88 KiB; some range length N*P*Q / (256 r / (K/64)), r = 1 .. 8, must divide P*Q and leave
 *     the ring's fill one step ahead of the MFMAs from every column a range can start in). */
/* The reduction operators with their launch shape chosen by the caller (same arguments, results
 * and errors as perf_softmax / perf_layernorm; every variant computes the same arithmetic, only
 * the summation tree differs with waves_per_row).  A knob left 0 keeps the library's rule; all
 * knobs 0, or a choice that cannot run the problem, returns UNSUPPORTED.  Only the 16-byte
 * aligned case has variants.
 *   perf_softmax_variant:
 *     waves_per_row  1 = a wavefront owns whole rows (cols <= 2048), rows_per_wave of them at a time:
 *                        1, 2, 4 or 8, with ceil(cols / 256) rounded up to a power of two times
 *                        rows_per_wave <= 16 (the lane's registers);
 *                    4 or 16 = a workgroup of that many wavefronts owns a row (cols <= 8192 / 32768),
 *                        rows_per_wave must be 0
 *     grid           workgroups to launch (they loop over the rows); 0 = one pass (waves_per_row 1)
 *                    or all wave slots of the chip (4, 16)
 *   perf_layernorm_variant:
 *     waves_per_row  1 (a wavefront per row: up to 16 chunks of 16 bytes per lane), 4 or 16 (a
 *                    workgroup per row, row in its registers: up to 32 KiB / 64 KiB (bf16) or 128 KiB
 *                    (f32) of input; gamma and beta 16-byte aligned)
 *     grid           workgroups to launch; 0 = the library's (1536 of four waves, or all wave slots) */
perf_status perf_softmax_variant(const void *x, void *y, int64_t rows, int64_t cols, int64_t ldx, int64_t ldy,
                                 perf_dtype x_dt, perf_dtype y_dt, float scale, int rows_per_wave,
                                 int waves_per_row, int64_t grid, perf_stream stream);
perf_status perf_layernorm_variant(const void *x, const void *gamma, const void *beta, void *y, float *mean_out,
                                   float *rstd_out, int64_t rows, int64_t cols, int64_t ldx, int64_t ldy, float eps,
                                   perf_dtype x_dt, perf_dtype param_dt, perf_dtype y_dt, int waves_per_row,
                                   int64_t grid, perf_stream stream);

perf_status perf_gemm_variant(const void *A, const void *B, void *C, int64_t M, int64_t N, int64_t K,
                              perf_layout la, int64_t lda, perf_layout lb, int64_t ldb, int64_t ldc,
                              int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC,
                              float alpha, perf_dtype ab_dt, perf_dtype c_dt, int tile, int kstep,
                              perf_stream stream);
perf_status perf_conv2d_variant(const void *x, const void *w, void *y, int64_t N, int64_t H, int64_t W,
                                int64_t C, int64_t K, int64_t R, int64_t S, int64_t stride_h,
                                int64_t stride_w, int64_t pad_h, int64_t pad_w, perf_dtype xw_dt,
                                perf_dtype y_dt, int variant, perf_stream stream);

/* Plain device-to-device streaming copy of `bytes` bytes (dst and src must not overlap).
 * It is the measured HBM ceiling the benchmark prints beside each bandwidth figure and
 * the known-size kernel against which profiler byte counters are scaled; it is not one
 * of the paper's operators.  Errors: NULL, SHAPE (bytes < 0), LAUNCH. */
perf_status perf_copy(const void *src, void *dst, int64_t bytes, perf_stream stream);

/* Streaming probe behind the benchmark's copy-ceiling study (not one of the paper's operators):
 * the copy kernel's access pattern with its knobs exposed, and its read and write halves alone.
 *   mode     0 = copy src -> dst, 1 = read src only (dst receives at most 16 bytes), 2 = write dst only
 *   bytes    a multiple of 16, >= 16; src and dst device, 16-byte aligned, at least `bytes` long
 *   unroll   16-byte vectors per thread and iteration: 1, 2, 4, 8 or 16
 *   threads  workgroup size: 64, 128, 256, 512 or 1024
 *   grid     0 = one pass per workgroup; otherwise that many workgroups, which loop over the data
 *   policy   bit 0 = non-temporal loads, bit 1 = non-temporal stores
 * Errors: NULL, SHAPE (bytes, mode, threads, grid or policy out of range), ALIGN, UNSUPPORTED
 * (unroll), LAUNCH. */
perf_status perf_stream_probe(const void *src, void *dst, int64_t bytes, int mode, int unroll, int threads,
                              int64_t grid, int policy, perf_stream stream);

/* Register-only bf16 MFMA loop, the measured matrix-core ceiling printed beside the GEMM and
 * convolution figures (not one of the paper's operators): 4096 wavefronts (1024 workgroups
 * of 256 threads) each issue iters * 32 v_mfma_f32_32x32x16_bf16 on 16 independent
 * accumulators, i.e. 4096 * iters * 32 * 32768 flop per call, with no memory access inside
 * the loop.  `sink` (device, at least 4096 floats, written once per wavefront) keeps the
 * result live.  Errors: NULL, SHAPE (iters < 1 or > 2^24), ALIGN, LAUNCH. */
perf_status perf_mfma_probe(float *sink, int64_t iters, perf_stream stream);
/* The same loop with a different pair of pseudo-random operand registers (values in [-1, 1))
 * for every accumulator, so that the multipliers toggle as they do in a GEMM on random data: the
 * clock the power management grants, and so the attainable rate, depends on the operand values.
 * Arguments and errors as perf_mfma_probe. */
perf_status perf_mfma_probe_random(float *sink, int64_t iters, perf_stream stream);

/* LDS read probes behind the convolution analysis (not one of the paper's operators): 256
 * workgroups of `waves` wavefronts (4, 8 or 16), every wavefront reading its own conflict-free
 * region.  with_mfma = 0: iters * 16 reads of bytes_per_lane (4, 8 or 16) bytes per lane, 16 in
 * flight; LDS bytes per clock and CU = waves * iters * 16 * 64 * bytes_per_lane / cycles.
 * with_mfma = 1 (bytes_per_lane 16): the weights-in-registers kernels' inner pattern, one
 * v_mfma_f32_32x32x16_bf16 plus the ds_read_b128 of the operand used nine MFMAs later,
 * iters * 36 of them; cycles / (iters * 36) against 32 is what that pattern costs a wavefront.
 * with_mfma = 2: the same with five dependent 32-bit multiply-adds behind each of 4 of the 36 MFMAs (vector
 * work hides behind an MFMA only for as long as the MFMA takes).
 *   cycles  device, one 64-bit value the caller has set to 0: raised (atomic max) to the shader cycles
 *           the slowest wavefront of workgroup 0 spent in the loop
 *   sink    device, one float, never written (keeps the reads live)
 * Errors: NULL, SHAPE (waves, bytes_per_lane, with_mfma, iters < 1 or > 2^24), UNSUPPORTED (with_mfma and
 * bytes_per_lane != 16), ALIGN, LAUNCH. */
perf_status perf_lds_probe(long long *cycles, float *sink, int waves, int bytes_per_lane, int with_mfma,
                           int64_t iters, perf_stream stream);

/* L2 -> CU feed probe behind the convolution and GEMM analysis (not one of the paper's operators): 256
 * workgroups of `waves` wavefronts (4 or 8) stream 1 KiB wave loads from a window of `span` bytes (a power
 * of two from 1 KiB to 1 GiB), the workgroup's own (shared = 0: window b of src for workgroup b) or one
 * window for all (shared = 1), iters * 8 loads per wavefront with eight more in flight; a window beyond the
 * L1's 32 KiB is served by the L2.  Bytes per clock and CU = waves * iters * 8192 / cycles.
 *   mode 0  buffer_load ... lds, whole KiB          mode 1  load to registers, then ds_write_b128
 *   mode 2  load to registers only                  mode 3  buffer_load ... lds in the slab convolution's
 *           row pattern (7 pixels x 8 lanes of 16 bytes, every ninth lane out of range)
 *   src     device, 16-byte aligned, src_bytes >= span (shared) or 256 * span; read only
 *   cycles  device, one 64-bit value the caller has set to 0: raised (atomic max) to the shader cycles the
 *           slowest wavefront of workgroup 0 spent in the loop
 *   sink    device, one float, never written for finite input (keeps the loads live)
 * Errors: NULL, SHAPE (waves, mode, shared, span, src_bytes, iters < 1 or > 2^14), ALIGN, LAUNCH. */
perf_status perf_feed_probe(const void *src, int64_t src_bytes, long long *cycles, float *sink, int waves, int mode,
                            int shared, int64_t span, int64_t iters, perf_stream stream);

/* Human-readable name of a status code; static storage, never freed. */
const char *perf_status_string(perf_status s);

/* Library version: major*10000 + minor*100 + patch. */
int perf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PERF_H */
