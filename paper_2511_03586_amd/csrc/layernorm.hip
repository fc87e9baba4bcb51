// LayerNorm over the last dimension for gfx950 ("layernorm" rows of the operator table,
// Section 4.3 of the paper; the mean -> variance -> scale -> shift staging is the one the
// paper describes for its batch-normalisation kernel, Section 4.3).
//
//  * layernorm_rows_kernel: a wavefront owns a whole row.  The row is read from HBM once
//    with 128-bit loads into registers.  Statistics are the corrected two-pass form, both
//    passes over registers: a provisional mean from the plain sum, then the first and
//    second moments of the data shifted by it (the first moment corrects the provisional
//    mean, the second gives the variance without cancellation).  Sums are reduced over the
//    64 lanes with a DPP / permlane butterfly (no LDS, no barrier per row).  A pairwise
//    Welford/Chan merge of per-lane (mean, M2) was measured less accurate: it rounds
//    per-lane means to fp32, which costs |mean|/sigma * 2^-24 per merge.  gamma and beta
//    are staged once per workgroup in LDS as fp32 and re-used for every row.
//  * norm_wide_kernel (wide_rows.h): rows beyond a wavefront's registers, one workgroup per
//    row, the row parked in LDS: still one read of HBM.
//  * layernorm_block_kernel: general fallback (any length, any alignment), one workgroup
//    per row, three passes over global memory with the same arithmetic.
#include "row_io.h"
#include "wide_rows.h"
#include "host_utils.h"

namespace perf {

constexpr int kLnThreads = 256;  // 256 threads x 1536 workgroups measured best on 8192x4096 bf16 (21.8 us; 22.4-23.3 us for 512 .. 4096)
constexpr int kLnWaves = kLnThreads / 64;

// XT, YT: element types of x and y; PT: element type of gamma/beta; NC: 16-byte chunks of
// the row held per lane (cols <= NC * 64 * E); EVEN: cols == NC * 64 * E exactly.
template <typename XT, typename PT, typename YT, int NC, bool EVEN>
__global__ __launch_bounds__(kLnThreads) void layernorm_rows_kernel(const XT *__restrict__ x,
                                                                    const PT *__restrict__ gamma,
                                                                    const PT *__restrict__ beta, YT *__restrict__ y,
                                                                    float *__restrict__ mean_out,
                                                                    float *__restrict__ rstd_out, int64_t rows,
                                                                    int cols, int64_t ldx, int64_t ldy, float eps)
{
    constexpr int E = Elem<XT>::kPerChunk;
    constexpr int NCH = NC * 64;  // chunks per (padded) row
    // gamma / beta as fp32, split in planes of 4 floats per chunk so that lane l reads
    // 16 bytes at stride 16: plane q of chunk c holds elements c*E + 4q .. c*E + 4q+3.
    extern __shared__ float4_t lds[];
    float4_t *g_lds = lds;                       // [E/4][NCH]
    float4_t *b_lds = lds + (E / 4) * NCH;       // [E/4][NCH]
    for (int i = threadIdx.x; i < (E / 4) * NCH; i += kLnThreads) {
        const int q = i / NCH, c = i % NCH;
        const int col = c * E + 4 * q;
        float4_t g = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
        if (col < cols) {  // cols is a multiple of E, so a chunk is entirely valid or not
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                g[e] = Elem<PT>::load1(gamma + col + e);
                b[e] = Elem<PT>::load1(beta + col + e);
            }
        }
        g_lds[i] = g;
        b_lds[i] = b;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * kLnWaves + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * kLnWaves;
    const float inv_cols = 1.0f / (float)cols;

    uint4_t raw[NC];
    auto load_row = [&](int64_t r) {
        const XT *xr = x + r * ldx;
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            const int c = (j * 64 + lane) * E;
            if (EVEN || c < cols)
                raw[j] = *reinterpret_cast<const uint4_t *>(xr + c);  // (plain loads measured 6 % faster here than non-temporal ones)
            else
                raw[j] = uint4_t{0u, 0u, 0u, 0u};
        }
    };
    if (wave < rows) load_row(wave);
    for (int64_t r = wave; r < rows; r += nwaves) {
        // Pass 1 (registers): provisional mean from the plain sum.
        float v[NC][E];
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            Elem<XT>::unpack(raw[j], v[j]);
#pragma unroll
            for (int e = 0; e < E; ++e) s += v[j][e];  // padding chunks hold zeros
        }
        // the raw registers are free again: the next row's loads fly during this row's arithmetic
        if (r + nwaves < rows) load_row(r + nwaves);
        const float mean0 = wave_allreduce(s, OpSum{}) * inv_cols;
        // Pass 2 (registers): shift by the provisional mean, then first and second moments
        // of the shifted data.  The shifted values are small, so neither moment cancels, and
        // the first moment corrects the rounding of mean0.
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            const bool valid = EVEN || (j * 64 + lane) * E < cols;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float d = valid ? v[j][e] - mean0 : 0.f;
                v[j][e] = d;
                s1 += d;
                s2 = __builtin_fmaf(d, d, s2);
            }
        }
        s1 = wave_allreduce(s1, OpSum{});
        s2 = wave_allreduce(s2, OpSum{});
        const float dm = s1 * inv_cols;
        const float mean = mean0 + dm;
        const float var = __builtin_fmaxf(__builtin_fmaf(-dm, dm, s2 * inv_cols), 0.f);
        const float rstd = 1.0f / __builtin_sqrtf(var + eps);
        if (lane == 0) {
            if (mean_out) mean_out[r] = mean;
            if (rstd_out) rstd_out[r] = rstd;
        }
        YT *yr = y + r * ldy;
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            const int ch = j * 64 + lane;
            if (EVEN || ch * E < cols) {
                float o[E];
#pragma unroll
                for (int q = 0; q < E / 4; ++q) {
                    const float4_t g = g_lds[q * NCH + ch];
                    const float4_t b = b_lds[q * NCH + ch];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        o[4 * q + e] = __builtin_fmaf((v[j][4 * q + e] - dm) * rstd, g[e], b[e]);
                }
                store_chunk<YT, E>(yr + ch * E, o);
            }
            // keeps the LDS reads of gamma / beta chunk by chunk; hoisted together they
            // double the register count and halve the occupancy
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// General fallback: one workgroup (256 threads) per row, scalar accesses, three passes.
__device__ __forceinline__ float block_sum_256(float v, float *red)
{
    v = wave_allreduce(v, OpSum{});
    __syncthreads();  // red may still be read from the previous use
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

template <typename XT, typename PT, typename YT>
__global__ __launch_bounds__(256) void layernorm_block_kernel(const XT *__restrict__ x, const PT *__restrict__ gamma,
                                                              const PT *__restrict__ beta, YT *__restrict__ y,
                                                              float *__restrict__ mean_out,
                                                              float *__restrict__ rstd_out, int64_t rows,
                                                              int64_t cols, int64_t ldx, int64_t ldy, float eps)
{
    __shared__ float red[4];
    const float inv_cols = 1.0f / (float)cols;
    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const XT *xr = x + r * ldx;
        YT *yr = y + r * ldy;
        float s = 0.f;
        for (int64_t c = threadIdx.x; c < cols; c += 256) s += Elem<XT>::load1(xr + c);
        const float mean0 = block_sum_256(s, red) * inv_cols;
        float s1 = 0.f, s2 = 0.f;
        for (int64_t c = threadIdx.x; c < cols; c += 256) {
            const float d = Elem<XT>::load1(xr + c) - mean0;
            s1 += d;
            s2 = __builtin_fmaf(d, d, s2);
        }
        const float dm = block_sum_256(s1, red) * inv_cols;
        const float var = __builtin_fmaxf(__builtin_fmaf(-dm, dm, block_sum_256(s2, red) * inv_cols), 0.f);
        const float rstd = 1.0f / __builtin_sqrtf(var + eps);
        if (threadIdx.x == 0) {
            if (mean_out) mean_out[r] = mean0 + dm;
            if (rstd_out) rstd_out[r] = rstd;
        }
        for (int64_t c = threadIdx.x; c < cols; c += 256) {
            const float d = Elem<XT>::load1(xr + c) - mean0;
            Elem<YT>::store1(yr + c, __builtin_fmaf((d - dm) * rstd, Elem<PT>::load1(gamma + c),
                                                     Elem<PT>::load1(beta + c)));
        }
    }
}

struct LnArgs {
    const void *x, *gamma, *beta;
    void *y;
    float *mean_out, *rstd_out;
    int64_t rows, cols, ldx, ldy;
    float eps;
    hipStream_t st;
    bool params_vec;  // gamma and beta are 16-byte aligned
    int waves_per_row;  // 0 = by shape; 1, 4, 16 = the caller's choice (perf_layernorm_variant)
    int64_t grid;       // 0 = by shape; else that many workgroups
    int failed;         // 0 = launched, 1 = a HIP call failed, 2 = the chosen kernel cannot run the rows
};

template <typename XT, typename PT, typename YT, int NC>
static void launch_rows_nc(const LnArgs &a)
{
    constexpr int E = Elem<XT>::kPerChunk;
    const size_t lds_bytes = (size_t)2 * (E / 4) * NC * 64 * sizeof(float4_t);
    int64_t blocks = (a.rows + kLnWaves - 1) / kLnWaves;
    const int64_t cap = a.grid > 0 ? a.grid : 1536;  // six workgroups per CU (two rounds of the three that are resident); waves then loop over rows
    if (blocks > cap) blocks = cap;
    const bool even = a.cols == (int64_t)NC * 64 * E;
    auto kern = even ? layernorm_rows_kernel<XT, PT, YT, NC, true> : layernorm_rows_kernel<XT, PT, YT, NC, false>;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kLnThreads), lds_bytes, a.st, (const XT *)a.x,
                       (const PT *)a.gamma, (const PT *)a.beta, (YT *)a.y, a.mean_out, a.rstd_out, a.rows, (int)a.cols,
                       a.ldx, a.ldy, a.eps);
}

template <typename XT, typename PT, typename YT>
static void launch_typed(LnArgs &a, bool vec_ok)
{
    constexpr int E = Elem<XT>::kPerChunk;
    const int64_t chunks = (a.cols + 64 * E - 1) / (64 * E);  // chunks per lane
    const bool variant = a.waves_per_row != 0 || a.grid != 0;
    if (variant && (!vec_ok || (a.waves_per_row == 1 && chunks > 16) || (a.waves_per_row > 1 && !a.params_vec))) {
        a.failed = 2;
        return;
    }
    if (vec_ok && chunks <= 16 && a.waves_per_row <= 1) {
        if (chunks <= 1) launch_rows_nc<XT, PT, YT, 1>(a);
        else if (chunks <= 2) launch_rows_nc<XT, PT, YT, 2>(a);
        else if (chunks <= 4) launch_rows_nc<XT, PT, YT, 4>(a);
        else if (chunks <= 8) launch_rows_nc<XT, PT, YT, 8>(a);
        else launch_rows_nc<XT, PT, YT, 16>(a);
    } else if (vec_ok && a.params_vec) {
        // longer rows: a workgroup per row, the row in its registers or parked in LDS (one read of HBM)
        a.failed = launch_norm_wide<XT, PT, YT, false>(a.x, a.gamma, a.beta, a.y, a.mean_out, a.rstd_out, a.rows, a.cols,
                                                       a.ldx, a.ldy, a.eps, a.st, a.waves_per_row, a.grid);
    } else {
        int64_t blocks = a.rows < 65536 ? a.rows : 65536;
        hipLaunchKernelGGL((layernorm_block_kernel<XT, PT, YT>), dim3((unsigned)blocks), dim3(256), 0, a.st,
                           (const XT *)a.x, (const PT *)a.gamma, (const PT *)a.beta, (YT *)a.y, a.mean_out, a.rstd_out,
                           a.rows, a.cols, a.ldx, a.ldy, a.eps);
    }
}

template <typename XT, typename PT>
static void launch_y(LnArgs &a, bool vec_ok, int y_dt)
{
    if (y_dt == PERF_F32) launch_typed<XT, PT, float>(a, vec_ok);
    else launch_typed<XT, PT, uint16_t>(a, vec_ok);
}

template <typename XT>
static void launch_p(LnArgs &a, bool vec_ok, int p_dt, int y_dt)
{
    if (p_dt == PERF_F32) launch_y<XT, float>(a, vec_ok, y_dt);
    else launch_y<XT, uint16_t>(a, vec_ok, y_dt);
}

}  // namespace perf

namespace perf {

static perf_status layernorm_impl(const void *x, const void *gamma, const void *beta, void *y, float *mean_out,
                                  float *rstd_out, int64_t rows, int64_t cols, int64_t ldx, int64_t ldy, float eps,
                                  int x_dt, int param_dt, int y_dt, int waves_per_row, int64_t grid, perf_stream stream)
{
    if (!x || !gamma || !beta || !y) return PERF_ERR_NULL;
    if (!dtype_ok(x_dt) || !dtype_ok(param_dt) || !dtype_ok(y_dt)) return PERF_ERR_DTYPE;
    if (rows < 1 || cols < 1 || ldx < cols || ldy < cols || !(eps >= 0.f) || !std::isfinite(eps)) return PERF_ERR_SHAPE;
    if (rows > (INT64_MAX / 4) / ldx || rows > (INT64_MAX / 4) / ldy) return PERF_ERR_SHAPE;
    if (grid < 0 || grid > kMaxGridX) return PERF_ERR_SHAPE;
    if (!aligned(x, dtype_size(x_dt)) || !aligned(y, dtype_size(y_dt)) || !aligned(gamma, dtype_size(param_dt)) ||
        !aligned(beta, dtype_size(param_dt)) || (mean_out && !aligned(mean_out, 4)) ||
        (rstd_out && !aligned(rstd_out, 4)))
        return PERF_ERR_ALIGN;

    const int64_t ex = 16 / dtype_size(x_dt);  // elements per 16-byte chunk of x
    // the register path needs whole 16-byte chunks of x and 16-byte aligned groups of y
    const bool vec_ok = cols % ex == 0 && ldx % ex == 0 && aligned(x, 16) && aligned(y, 16) &&
                        (ldy * dtype_size(y_dt)) % 16 == 0;
    LnArgs a{x, gamma, beta, y, mean_out, rstd_out, rows, cols, ldx, ldy, eps, static_cast<hipStream_t>(stream),
             aligned(gamma, 16) && aligned(beta, 16), waves_per_row, grid, 0};
    if (x_dt == PERF_F32) launch_p<float>(a, vec_ok, param_dt, y_dt);
    else launch_p<uint16_t>(a, vec_ok, param_dt, y_dt);
    if (a.failed == 2) return PERF_ERR_UNSUPPORTED;
    return a.failed ? PERF_ERR_LAUNCH : launch_status();
}

}  // namespace perf

extern "C" perf_status perf_layernorm(const void *x, const void *gamma, const void *beta, void *y, float *mean_out,
                                      float *rstd_out, int64_t rows, int64_t cols, int64_t ldx, int64_t ldy, float eps,
                                      perf_dtype x_dt, perf_dtype param_dt, perf_dtype y_dt, perf_stream stream)
{
    return perf::layernorm_impl(x, gamma, beta, y, mean_out, rstd_out, rows, cols, ldx, ldy, eps, x_dt, param_dt, y_dt, 0,
                                0, stream);
}

extern "C" perf_status perf_layernorm_variant(const void *x, const void *gamma, const void *beta, void *y,
                                              float *mean_out, float *rstd_out, int64_t rows, int64_t cols, int64_t ldx,
                                              int64_t ldy, float eps, perf_dtype x_dt, perf_dtype param_dt,
                                              perf_dtype y_dt, int waves_per_row, int64_t grid, perf_stream stream)
{
    if ((waves_per_row != 0 && waves_per_row != 1 && waves_per_row != 4 && waves_per_row != 16) ||
        (waves_per_row == 0 && grid == 0))
        return PERF_ERR_UNSUPPORTED;
    return perf::layernorm_impl(x, gamma, beta, y, mean_out, rstd_out, rows, cols, ldx, ldy, eps, x_dt, param_dt, y_dt,
                                waves_per_row, grid, stream);
}
