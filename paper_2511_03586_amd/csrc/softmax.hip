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
//  * softmax_block_kernel: general fallback, one 256-thread workgroup per row, any
//    length or alignment; a streaming (max, sum) pair per thread is merged through LDS,
//    and the row is kept in LDS when it fits so HBM is still read once.
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

// General fallback: one workgroup per row, scalar accesses.
constexpr int kBlockCache = 12288;  // floats of a row kept in LDS (48 KiB)

__global__ __launch_bounds__(256) void softmax_block_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                            int64_t rows, int64_t cols, int64_t ldx, int64_t ldy,
                                                            ExpConst k)
{
    __shared__ float cache[kBlockCache];
    __shared__ float red_m[4], red_z[4];
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;

    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const float *xr = x + r * ldx;
        float *yr = y + r * ldy;
        // streaming (max, sum): s always holds sum exp(c*(x - m)) for the current m
        float m = -FLT_MAX, s = 0.f;
        for (int64_t c = tid; c < cols; c += 256) {
            float v = xr[c] * k.sign;
            if (c < kBlockCache) cache[c] = v;
            if (v > m) {
                s *= exp_scaled(m - v, k.c_hi, k.c_lo);
                m = v;
            }
            s += exp_scaled(v - m, k.c_hi, k.c_lo);
        }
        float wm = wave_allreduce(m, OpMax{});
        s *= exp_scaled(m - wm, k.c_hi, k.c_lo);
        s = wave_allreduce(s, OpSum{});
        if (lane == 0) {
            red_m[wid] = wm;
            red_z[wid] = s;
        }
        __syncthreads();
        float gm = __builtin_fmaxf(__builtin_fmaxf(red_m[0], red_m[1]), __builtin_fmaxf(red_m[2], red_m[3]));
        float z = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) z += red_z[w] * exp_scaled(red_m[w] - gm, k.c_hi, k.c_lo);
        const float inv = 1.0f / z;
        for (int64_t c = tid; c < cols; c += 256) {
            float v = c < kBlockCache ? cache[c] : xr[c] * k.sign;
            yr[c] = exp_scaled(v - gm, k.c_hi, k.c_lo) * inv;
        }
        __syncthreads();  // cache and red_* are reused by the next row
    }
}

template <int NV, int RPW>
static void launch_rows(const float *x, float *y, int64_t rows, int cols, int64_t ldx, int64_t ldy, ExpConst k,
                        hipStream_t st)
{
    int64_t blocks = (rows + 4 * RPW - 1) / (4 * RPW);
    if (blocks > 256 * 64) blocks = 256 * 64;  // then waves loop over rows
    hipLaunchKernelGGL((softmax_rows_kernel<NV, RPW>), dim3((unsigned)blocks), dim3(256), 0, st, x, y, rows, cols, ldx,
                       ldy, k);
}

}  // namespace perf

extern "C" perf_status perf_softmax(const void *x, void *y, int64_t rows, int64_t cols, int64_t ldx, int64_t ldy,
                                    perf_dtype x_dt, perf_dtype y_dt, float scale, perf_stream stream)
{
    using namespace perf;
    if (!x || !y) return PERF_ERR_NULL;
    if (!dtype_ok(x_dt) || !dtype_ok(y_dt)) return PERF_ERR_DTYPE;
    if (rows < 1 || cols < 1 || ldx < cols || ldy < cols || !std::isfinite(scale)) return PERF_ERR_SHAPE;
    if (rows > (INT64_MAX / 4) / ldx || rows > (INT64_MAX / 4) / ldy) return PERF_ERR_SHAPE;
    if (x_dt != PERF_F32 || y_dt != PERF_F32) return PERF_ERR_UNSUPPORTED;
    if (!aligned(x, 4) || !aligned(y, 4)) return PERF_ERR_ALIGN;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const float *xp = static_cast<const float *>(x);
    float *yp = static_cast<float *>(y);
    const ExpConst k = make_exp_const(scale);
    const bool vec_ok = cols <= 2048 && cols % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0 && aligned(x, 16) && aligned(y, 16);
    if (vec_ok) {
        const int c = (int)cols;
        if (c <= 256) launch_rows<1, 8>(xp, yp, rows, c, ldx, ldy, k, st);
        else if (c <= 512) launch_rows<2, 4>(xp, yp, rows, c, ldx, ldy, k, st);
        else if (c <= 1024) launch_rows<4, 2>(xp, yp, rows, c, ldx, ldy, k, st);
        else launch_rows<8, 1>(xp, yp, rows, c, ldx, ldy, k, st);
    } else {
        int64_t blocks = rows < 256 * 256 ? rows : 256 * 256;
        hipLaunchKernelGGL(softmax_block_kernel, dim3((unsigned)blocks), dim3(256), 0, st, xp, yp, rows, cols, ldx, ldy,
                           k);
    }
    return launch_status();
}
