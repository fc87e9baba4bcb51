// Row softmax for gfx950 (Fig. "Softmax kernel representations", Section 2.1 of the
// paper; "softmax" row of the operator table, Section 4.3).
//
// The paper reaches a fast softmax by fusing the max / exp / sum / divide scopes and
// dropping the temporaries' row dimension (Fig. "Program transformation example").  The
// same end state is written here directly for wave64 hardware: a row is read from HBM
// once with 128-bit loads, lives in registers, and is written once.
//
//  * softmax_rows_kernel: one wavefront owns RPW whole rows at a time (cols <= 2048,
//    16-byte aligned).  Reductions are DPP / permlane butterflies, no LDS, no barrier.
//  * softmax_wgrow_kernel: rows of 8 .. 128 KiB, one workgroup (4 or 16 waves) per row, the
//    row in the workgroup's registers, the next row's loads in flight meanwhile.
//  * softmax_wide_kernel: still longer or unaligned rows, one workgroup per row:
//    the row goes to LDS (up to 144 KiB, 16-byte accesses when aligned) and is read from HBM
//    once; what a longer row has beyond that is read twice.
#include <atomic>
#include "softmax_math.h"
#include "host_utils.h"

namespace perf {

template <int NV, int RPW>
__global__ __launch_bounds__(256) void softmax_rows_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                           int64_t rows, int cols, int64_t ldx, int64_t ldy,
                                                           ExpConst k)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;

    for (int64_t r0 = wave * RPW; r0 < rows; r0 += nwaves * RPW) {
        float4_t v[RPW][NV];
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int64_t r = r0 + i;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int c = (j * 64 + lane) * 4;
                if (r < rows && c < cols)
                    v[i][j] = __builtin_nontemporal_load(reinterpret_cast<const float4_t *>(x + r * ldx + c));
                else
                    v[i][j] = float4_t{-FLT_MAX, -FLT_MAX, -FLT_MAX, -FLT_MAX} * k.sign;
            }
        }
#pragma unroll
        for (int i = 0; i < RPW; ++i) {
            const int64_t r = r0 + i;
            float m = -FLT_MAX;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                v[i][j] *= k.sign;  // exact; turns the scale < 0 case into a max problem
                m = __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fmaxf(v[i][j][0], v[i][j][1]),
                                                       __builtin_fmaxf(v[i][j][2], v[i][j][3])));
            }
            m = wave_allreduce(m, OpMax{});
            float z = 0.f;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const bool valid = (j * 64 + lane) * 4 < cols;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float t = exp_scaled(v[i][j][e] - m, k.c_hi, k.c_lo);
                    v[i][j][e] = valid ? t : 0.f;
                    z += v[i][j][e];
                }
            }
            z = wave_allreduce(z, OpSum{});
            const float inv = 1.0f / z;
            if (r < rows) {
#pragma unroll
                for (int j = 0; j < NV; ++j) {
                    const int c = (j * 64 + lane) * 4;
                    if (c < cols)
                        __builtin_nontemporal_store(v[i][j] * inv, reinterpret_cast<float4_t *>(y + r * ldy + c));
                }
            }
        }
    }
}

// Rows that do not fit a wavefront's registers: one workgroup of THREADS per row.  The row
// is read from HBM once into LDS (its first `cap` floats; 16-byte accesses when VEC), the
// exponentials replace it there, and the normalised row is written from there.  What lies
// beyond `cap` (rows longer than the LDS) is read a second time instead.  Any length, any
// alignment (VEC = false: element accesses).
template <int THREADS>
__device__ __forceinline__ float block_reduce_max(float v, float *red)
{
    v = wave_allreduce(v, OpMax{});
    __syncthreads();  // red may still be read from its previous use
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int w = 1; w < THREADS / 64; ++w) r = __builtin_fmaxf(r, red[w]);
    return r;
}
template <int THREADS>
__device__ __forceinline__ float block_reduce_sum(float v, float *red)
{
    v = wave_allreduce(v, OpSum{});
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = 0.f;
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) r += red[w];  // fixed order: bit-identical reruns
    return r;
}

// Rows of 8 KiB .. 128 KiB: one workgroup of THREADS per row, the row in the workgroup's
// registers (NV 16-byte vectors per thread), LDS only for the two cross-wave reductions.  The
// next row's loads are issued before this row's arithmetic, so a workgroup always has a row in
// flight and reads, exponentials and writes of different rows overlap.
template <int THREADS, int NV>
__global__ __launch_bounds__(THREADS) void softmax_wgrow_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                int64_t rows, int cols, int64_t ldx, int64_t ldy,
                                                                ExpConst k)
{
    __shared__ float red[THREADS / 64];
    const int tid = threadIdx.x, n4 = cols / 4;
    float4_t cur[NV], nxt[NV];
    auto load_row = [&](float4_t (&v)[NV], int64_t r) {
        const float4_t *xr = reinterpret_cast<const float4_t *>(x + r * ldx);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = j * THREADS + tid;
            if (c < n4) v[j] = __builtin_nontemporal_load(xr + c);
            else v[j] = float4_t{-FLT_MAX, -FLT_MAX, -FLT_MAX, -FLT_MAX} * k.sign;
        }
    };
    int64_t r = blockIdx.x;
    if (r < rows) load_row(cur, r);
    for (; r < rows; r += gridDim.x) {
        if (r + gridDim.x < rows) load_row(nxt, r + gridDim.x);
        float m = -FLT_MAX;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            cur[j] *= k.sign;  // exact; turns the scale < 0 case into a max problem
            m = __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fmaxf(cur[j][0], cur[j][1]), __builtin_fmaxf(cur[j][2], cur[j][3])));
        }
        m = block_reduce_max<THREADS>(m, red);
        float z = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const bool valid = j * THREADS + tid < n4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float t = exp_scaled(cur[j][e] - m, k.c_hi, k.c_lo);
                cur[j][e] = valid ? t : 0.f;
                z += cur[j][e];
            }
        }
        const float inv = 1.0f / block_reduce_sum<THREADS>(z, red);
        float4_t *yr = reinterpret_cast<float4_t *>(y + r * ldy);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = j * THREADS + tid;
            if (c < n4) __builtin_nontemporal_store(cur[j] * inv, yr + c);
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) cur[j] = nxt[j];
    }
}

template <int THREADS, int NV>
static perf_status launch_wgrow(const float *x, float *y, int64_t rows, int cols, int64_t ldx, int64_t ldy, ExpConst k,
                                hipStream_t st, int64_t grid = 0)
{
    // 16 workgroups per CU (more than are resident: the variant search measured 182 us against
    // 200 with just the resident ones on 8192 x 16384)
    int64_t blocks = rows < 256 * 16 ? rows : 256 * 16;
    if (grid > 0) blocks = grid < rows ? grid : rows;
    hipLaunchKernelGGL((softmax_wgrow_kernel<THREADS, NV>), dim3((unsigned)blocks), dim3(THREADS), 0, st, x, y, rows, cols,
                       ldx, ldy, k);
    return launch_status();
}

template <int THREADS, bool VEC>
__global__ __launch_bounds__(THREADS) void softmax_wide_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                               int64_t rows, int64_t cols, int64_t ldx, int64_t ldy,
                                                               ExpConst k, int64_t cap)
{
    extern __shared__ float4_t cache4[];  // cap floats (cap is a multiple of 4)
    float *const cache = reinterpret_cast<float *>(cache4);
    __shared__ float red[THREADS / 64];
    const int tid = threadIdx.x;
    constexpr int kU = 4;  // independent loads in flight per thread

    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const float *xr = x + r * ldx;
        float *yr = y + r * ldy;
        float m = -FLT_MAX;
        if constexpr (VEC) {
            const float4_t *xr4 = reinterpret_cast<const float4_t *>(xr);
            float4_t *yr4 = reinterpret_cast<float4_t *>(yr);
            const int64_t n4 = cols / 4, cap4 = cap / 4;
            auto take = [&](int64_t c, float4_t v) {
                v *= k.sign;  // exact; turns the scale < 0 case into a max problem
                if (c < cap4) cache4[c] = v;
                m = __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fmaxf(v[0], v[1]), __builtin_fmaxf(v[2], v[3])));
            };
            int64_t c = tid;
            for (; c + (kU - 1) * THREADS < n4; c += kU * THREADS) {
                float4_t v[kU];
#pragma unroll
                for (int u = 0; u < kU; ++u) v[u] = __builtin_nontemporal_load(xr4 + c + u * THREADS);
#pragma unroll
                for (int u = 0; u < kU; ++u) take(c + u * THREADS, v[u]);
            }
            for (; c < n4; c += THREADS) take(c, __builtin_nontemporal_load(xr4 + c));
            m = block_reduce_max<THREADS>(m, red);
            float z = 0.f;
            for (c = tid; c < n4; c += THREADS) {
                float4_t v = c < cap4 ? cache4[c] : xr4[c] * k.sign;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] = exp_scaled(v[e] - m, k.c_hi, k.c_lo);
                    z += v[e];
                }
                if (c < cap4) cache4[c] = v;
            }
            const float inv = 1.0f / block_reduce_sum<THREADS>(z, red);
            for (c = tid; c < n4; c += THREADS) {
                float4_t v;
                if (c < cap4) {
                    v = cache4[c];
                } else {
                    v = xr4[c] * k.sign;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = exp_scaled(v[e] - m, k.c_hi, k.c_lo);
                }
                __builtin_nontemporal_store(v * inv, yr4 + c);
            }
        } else {
            for (int64_t c = tid; c < cols; c += THREADS) {
                const float v = xr[c] * k.sign;
                if (c < cap) cache[c] = v;
                m = __builtin_fmaxf(m, v);
            }
            m = block_reduce_max<THREADS>(m, red);
            float z = 0.f;
            for (int64_t c = tid; c < cols; c += THREADS) {
                const float e = exp_scaled((c < cap ? cache[c] : xr[c] * k.sign) - m, k.c_hi, k.c_lo);
                if (c < cap) cache[c] = e;
                z += e;
            }
            const float inv = 1.0f / block_reduce_sum<THREADS>(z, red);
            for (int64_t c = tid; c < cols; c += THREADS)
                yr[c] = (c < cap ? cache[c] : exp_scaled(xr[c] * k.sign - m, k.c_hi, k.c_lo)) * inv;
        }
        __syncthreads();  // the cache is reused by the next row
    }
}

constexpr int64_t kWideLdsBytes = 144 * 1024;  // of the CU's 160 KiB; rows up to 36864 floats are read once

template <int THREADS, bool VEC>
static perf_status launch_wide(const float *x, float *y, int64_t rows, int64_t cols, int64_t ldx, int64_t ldy, ExpConst k,
                               hipStream_t st)
{
    int64_t cap = (cols + 3) / 4 * 4;
    if (cap * 4 > kWideLdsBytes) cap = kWideLdsBytes / 4;
    const size_t lds = (size_t)cap * 4;
    auto kern = softmax_wide_kernel<THREADS, VEC>;
    static std::atomic<bool> attr_done{false};  // the dynamic-LDS cap is a per-function, idempotent setting
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)kWideLdsBytes) != hipSuccess)
            return PERF_ERR_LAUNCH;
        attr_done = true;
    }
    // as many workgroups per CU as LDS and wave slots allow, at most eight rounds of rows per launch
    int64_t per_cu = (160 * 1024) / (int64_t)(lds + 256);
    const int64_t by_waves = 2048 / THREADS;
    per_cu = per_cu < 1 ? 1 : per_cu > by_waves ? by_waves : per_cu;
    int64_t blocks = rows < 256 * per_cu ? rows : 256 * per_cu;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(THREADS), lds, st, x, y, rows, cols, ldx, ldy, k, cap);
    return launch_status();
}

template <int NV, int RPW>
static void launch_rows(const float *x, float *y, int64_t rows, int cols, int64_t ldx, int64_t ldy, ExpConst k,
                        hipStream_t st, int64_t grid = 0)
{
    int64_t blocks = (rows + 4 * RPW - 1) / (4 * RPW);
    // (one pass up to 256K workgroups: 167.5 us against 170.8 on 131072 x 1024 with waves looping over two rows each)
    if (blocks > 256 * 1024) blocks = 256 * 1024;  // then waves loop over rows
    if (grid > 0 && grid < blocks) blocks = grid;  // (a caller's choice of a persistent grid)
    hipLaunchKernelGGL((softmax_rows_kernel<NV, RPW>), dim3((unsigned)blocks), dim3(256), 0, st, x, y, rows, cols, ldx,
                       ldy, k);
}

}  // namespace perf

namespace perf {

// rows_per_wave / waves_per_row / grid: 0 = the library's shape rules; otherwise the caller's
// choice (perf_softmax_variant), UNSUPPORTED if that kernel cannot run the problem.
static perf_status softmax_impl(const void *x, void *y, int64_t rows, int64_t cols, int64_t ldx, int64_t ldy, int x_dt,
                                int y_dt, float scale, int rows_per_wave, int waves_per_row, int64_t grid,
                                perf_stream stream)
{
    if (!x || !y) return PERF_ERR_NULL;
    if (!dtype_ok(x_dt) || !dtype_ok(y_dt)) return PERF_ERR_DTYPE;
    if (rows < 1 || cols < 1 || ldx < cols || ldy < cols || !std::isfinite(scale)) return PERF_ERR_SHAPE;
    if (rows > (INT64_MAX / 4) / ldx || rows > (INT64_MAX / 4) / ldy) return PERF_ERR_SHAPE;
    if (grid < 0 || grid > kMaxGridX) return PERF_ERR_SHAPE;
    if (x_dt != PERF_F32 || y_dt != PERF_F32) return PERF_ERR_UNSUPPORTED;
    if (!aligned(x, 4) || !aligned(y, 4)) return PERF_ERR_ALIGN;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const float *xp = static_cast<const float *>(x);
    float *yp = static_cast<float *>(y);
    const ExpConst k = make_exp_const(scale);
    const bool vec = cols % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0 && aligned(x, 16) && aligned(y, 16);
    const bool variant = rows_per_wave != 0 || waves_per_row != 0 || grid != 0;
    if (variant && !vec) return PERF_ERR_UNSUPPORTED;  // the element-access path has no knobs
    if (waves_per_row == 0) waves_per_row = cols <= 2048 ? 1 : cols <= 8192 ? 4 : cols <= 32768 ? 16 : -1;

    if (vec && waves_per_row == 1) {
        // a wavefront per row, rows_per_wave rows at a time: NV 16-byte vectors per lane and row, at
        // most 16 vectors (64 registers) per lane in all
        const int c = (int)cols;
        const int nv = c <= 256 ? 1 : c <= 512 ? 2 : c <= 1024 ? 4 : 8;
        if (cols > 2048) return PERF_ERR_UNSUPPORTED;
        // the library's rule, from the variant search: 4 vectors per lane in flight (131072 x 1024:
        // 171 us against 174.5 with 8; 262144 x 512: 171 against 176); problems of less than 256 MiB
        // take one row per wave on a persistent grid of 16 workgroups per CU (24576 x 512: 17.8 us
        // against 19.3)
        if (rows_per_wave == 0) {
            const bool small = rows * cols * 8 < (int64_t(256) << 20);
            rows_per_wave = small ? 1 : nv >= 4 ? 1 : 4 / nv;
            if (small && grid == 0) grid = 256 * 16;
        }
#define PERF_SM_ROWS(NV, RPW)                                        \
    if (nv == NV && rows_per_wave == RPW) {                          \
        launch_rows<NV, RPW>(xp, yp, rows, c, ldx, ldy, k, st, grid); \
        return launch_status();                                      \
    }
        PERF_SM_ROWS(1, 1) PERF_SM_ROWS(1, 2) PERF_SM_ROWS(1, 4) PERF_SM_ROWS(1, 8)
        PERF_SM_ROWS(2, 1) PERF_SM_ROWS(2, 2) PERF_SM_ROWS(2, 4) PERF_SM_ROWS(2, 8)
        PERF_SM_ROWS(4, 1) PERF_SM_ROWS(4, 2) PERF_SM_ROWS(4, 4)
        PERF_SM_ROWS(8, 1) PERF_SM_ROWS(8, 2)
#undef PERF_SM_ROWS
        return PERF_ERR_UNSUPPORTED;
    }
    if (vec && (waves_per_row == 4 || waves_per_row == 16)) {
        // a workgroup per row, the row in its registers (at most 8 vectors per thread)
        if (rows_per_wave != 0) return PERF_ERR_UNSUPPORTED;
        const int64_t threads = 64 * waves_per_row;
        if (cols > threads * 8 * 4) return PERF_ERR_UNSUPPORTED;
        const int c = (int)cols;
        const bool small = cols <= threads * 4 * 4;
        if (waves_per_row == 4) return small ? launch_wgrow<256, 4>(xp, yp, rows, c, ldx, ldy, k, st, grid)
                                             : launch_wgrow<256, 8>(xp, yp, rows, c, ldx, ldy, k, st, grid);
        return small ? launch_wgrow<1024, 4>(xp, yp, rows, c, ldx, ldy, k, st, grid)
                     : launch_wgrow<1024, 8>(xp, yp, rows, c, ldx, ldy, k, st, grid);
    }
    if (variant) return PERF_ERR_UNSUPPORTED;
    // rows beyond 128 KiB, or nothing aligned: a workgroup per row through LDS
    if (cols > 8192) return vec ? launch_wide<1024, true>(xp, yp, rows, cols, ldx, ldy, k, st)
                                : launch_wide<1024, false>(xp, yp, rows, cols, ldx, ldy, k, st);
    return vec ? launch_wide<256, true>(xp, yp, rows, cols, ldx, ldy, k, st)
               : launch_wide<256, false>(xp, yp, rows, cols, ldx, ldy, k, st);
}

}  // namespace perf

extern "C" perf_status perf_softmax(const void *x, void *y, int64_t rows, int64_t cols, int64_t ldx, int64_t ldy,
                                    perf_dtype x_dt, perf_dtype y_dt, float scale, perf_stream stream)
{
    return perf::softmax_impl(x, y, rows, cols, ldx, ldy, x_dt, y_dt, scale, 0, 0, 0, stream);
}

extern "C" perf_status perf_softmax_variant(const void *x, void *y, int64_t rows, int64_t cols, int64_t ldx,
                                            int64_t ldy, perf_dtype x_dt, perf_dtype y_dt, float scale,
                                            int rows_per_wave, int waves_per_row, int64_t grid, perf_stream stream)
{
    if (rows_per_wave < 0 || waves_per_row < 0 || (rows_per_wave == 0 && waves_per_row == 0 && grid == 0))
        return PERF_ERR_UNSUPPORTED;
    return perf::softmax_impl(x, y, rows, cols, ldx, ldy, x_dt, y_dt, scale, rows_per_wave, waves_per_row, grid, stream);
}
