// LayerNorm and RMS norm for rows that do not fit a wavefront's registers ("layernorm" and
// "rmsnorm" rows of the operator table, Section 4.3 of the paper): one workgroup per row.
// norm_wgrow_kernel keeps rows of up to 128 KiB in the workgroup's registers; norm_wide_kernel
// takes longer ones: the row is read from HBM once, 16 bytes per lane, and parked in LDS as it
// came (raw fp32 or bf16 chunks); the statistics (the corrected two-pass form of the register kernels) and the
// affine step read it from there.  Chunks beyond the LDS capacity (`cap` chunks; rows longer
// than 144 KiB) are read from memory again in the later passes instead.
#pragma once
#include "row_io.h"

namespace perf {

constexpr int64_t kWideRowLdsBytes = 144 * 1024;

template <int THREADS>
__device__ __forceinline__ float wide_block_sum(float v, float *red)
{
    v = wave_allreduce(v, OpSum{});
    __syncthreads();  // red may still be read from its previous use
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = 0.f;
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) r += red[w];  // fixed order: bit-identical reruns
    return r;
}

// E parameters starting at element `col` (a multiple of E; p is 16-byte aligned) as fp32
template <typename PT, int E>
__device__ __forceinline__ void load_params(const PT *p, int64_t col, float *out)
{
    if constexpr (sizeof(PT) == 4) {
#pragma unroll
        for (int q = 0; q < E / 4; ++q) {
            const float4_t g = *reinterpret_cast<const float4_t *>(p + col + 4 * q);
#pragma unroll
            for (int e = 0; e < 4; ++e) out[4 * q + e] = g[e];
        }
    } else if constexpr (E == 8) {
        Elem<uint16_t>::unpack(*reinterpret_cast<const uint4_t *>(p + col), out);
    } else {
        const uint2_t g = *reinterpret_cast<const uint2_t *>(p + col);
        out[0] = bf16_lo(g[0]);
        out[1] = bf16_hi(g[0]);
        out[2] = bf16_lo(g[1]);
        out[3] = bf16_hi(g[1]);
    }
}

// RMS = false: y = (x - mean) * rstd * gamma + beta, stat0 = mean, stat1 = rstd.
// RMS = true:  y = x * rrms * gamma (beta unused), stat1 = rrms.
// cols is a multiple of E; x, y rows and gamma / beta are 16-byte aligned (the host checks).
template <typename XT, typename PT, typename YT, int THREADS, bool RMS>
__global__ __launch_bounds__(THREADS) void norm_wide_kernel(const XT *__restrict__ x, const PT *__restrict__ gamma,
                                                            const PT *__restrict__ beta, YT *__restrict__ y,
                                                            float *__restrict__ stat0, float *__restrict__ stat1,
                                                            int64_t rows, int64_t cols, int64_t ldx, int64_t ldy, float eps,
                                                            int64_t cap)
{
    constexpr int E = Elem<XT>::kPerChunk;
    constexpr int kU = 4;  // independent loads in flight per thread
    extern __shared__ uint4_t row_cache[];  // cap chunks
    __shared__ float red[THREADS / 64];
    const int tid = threadIdx.x;
    const int64_t nch = cols / E;
    const float inv_cols = 1.0f / (float)cols;

    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const uint4_t *xr = reinterpret_cast<const uint4_t *>(x + r * ldx);
        YT *yr = y + r * ldy;
        auto chunk = [&](int64_t c) { return c < cap ? row_cache[c] : xr[c]; };
        // pass 1: HBM -> LDS, plain sum (LayerNorm) or sum of squares (RMS norm)
        float s = 0.f;
        auto take = [&](int64_t c, uint4_t raw) {
            if (c < cap) row_cache[c] = raw;
            float v[E];
            Elem<XT>::unpack(raw, v);
#pragma unroll
            for (int e = 0; e < E; ++e) s = RMS ? __builtin_fmaf(v[e], v[e], s) : s + v[e];
        };
        int64_t c = tid;
        for (; c + (kU - 1) * THREADS < nch; c += kU * THREADS) {
            uint4_t raw[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) raw[u] = __builtin_nontemporal_load(xr + c + u * THREADS);
#pragma unroll
            for (int u = 0; u < kU; ++u) take(c + u * THREADS, raw[u]);
        }
        for (; c < nch; c += THREADS) take(c, __builtin_nontemporal_load(xr + c));
        s = wide_block_sum<THREADS>(s, red);
        float shift = 0.f, scale;
        if constexpr (RMS) {
            scale = 1.0f / __builtin_sqrtf(s * inv_cols + eps);
            if (tid == 0 && stat1) stat1[r] = scale;
        } else {
            // pass 2: first and second moments of the data shifted by the provisional mean
            const float mean0 = s * inv_cols;
            float s1 = 0.f, s2 = 0.f;
            for (c = tid; c < nch; c += THREADS) {
                float v[E];
                Elem<XT>::unpack(chunk(c), v);
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float d = v[e] - mean0;
                    s1 += d;
                    s2 = __builtin_fmaf(d, d, s2);
                }
            }
            s1 = wide_block_sum<THREADS>(s1, red);
            s2 = wide_block_sum<THREADS>(s2, red);
            const float dm = s1 * inv_cols;
            const float var = __builtin_fmaxf(__builtin_fmaf(-dm, dm, s2 * inv_cols), 0.f);
            scale = 1.0f / __builtin_sqrtf(var + eps);
            shift = mean0;
            if (tid == 0) {
                if (stat0) stat0[r] = mean0 + dm;
                if (stat1) stat1[r] = scale;
            }
            // (v - mean0 - dm) * rstd, with the two subtractions kept apart as in the register kernel
            for (c = tid; c < nch; c += THREADS) {
                float v[E], g[E], b[E], o[E];
                Elem<XT>::unpack(chunk(c), v);
                load_params<PT, E>(gamma, c * E, g);
                load_params<PT, E>(beta, c * E, b);
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] = __builtin_fmaf(((v[e] - shift) - dm) * scale, g[e], b[e]);
                store_chunk<YT, E>(yr + c * E, o);
            }
        }
        if constexpr (RMS) {
            for (c = tid; c < nch; c += THREADS) {
                float v[E], g[E], o[E];
                Elem<XT>::unpack(chunk(c), v);
                load_params<PT, E>(gamma, c * E, g);
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] = v[e] * scale * g[e];
                store_chunk<YT, E>(yr + c * E, o);
            }
        }
        __syncthreads();  // the cache is reused by the next row
    }
}

// Rows of 16 .. 128 KiB of input: one workgroup of THREADS per row, the row in the workgroup's
// registers (NC 16-byte chunks per thread), LDS only for the cross-wave sums.  The next row's
// loads are issued as soon as this row is unpacked, so a workgroup always has a row in flight.
template <typename XT, typename PT, typename YT, int THREADS, int NC, bool RMS>
__global__ __launch_bounds__(THREADS) void norm_wgrow_kernel(const XT *__restrict__ x, const PT *__restrict__ gamma,
                                                             const PT *__restrict__ beta, YT *__restrict__ y,
                                                             float *__restrict__ stat0, float *__restrict__ stat1,
                                                             int64_t rows, int cols, int64_t ldx, int64_t ldy, float eps)
{
    constexpr int E = Elem<XT>::kPerChunk;
    __shared__ float red[THREADS / 64];
    const int tid = threadIdx.x, nch = cols / E;
    const float inv_cols = 1.0f / (float)cols;
    uint4_t raw[NC];
    auto load_row = [&](int64_t r) {
        const uint4_t *xr = reinterpret_cast<const uint4_t *>(x + r * ldx);
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            const int c = j * THREADS + tid;
            raw[j] = c < nch ? __builtin_nontemporal_load(xr + c) : uint4_t{0u, 0u, 0u, 0u};
        }
    };
    int64_t r = blockIdx.x;
    if (r < rows) load_row(r);
    for (; r < rows; r += gridDim.x) {
        float v[NC][E];
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            Elem<XT>::unpack(raw[j], v[j]);
#pragma unroll
            for (int e = 0; e < E; ++e) s = RMS ? __builtin_fmaf(v[j][e], v[j][e], s) : s + v[j][e];  // padding chunks hold zeros
        }
        if (r + gridDim.x < rows) load_row(r + gridDim.x);  // flies during this row's arithmetic and stores
        s = wide_block_sum<THREADS>(s, red);
        float scale, dm = 0.f;
        if constexpr (RMS) {
            scale = 1.0f / __builtin_sqrtf(s * inv_cols + eps);
            if (tid == 0 && stat1) stat1[r] = scale;
        } else {
            const float mean0 = s * inv_cols;
            float s1 = 0.f, s2 = 0.f;
#pragma unroll
            for (int j = 0; j < NC; ++j) {
                const bool valid = j * THREADS + tid < nch;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float d = valid ? v[j][e] - mean0 : 0.f;
                    v[j][e] = d;
                    s1 += d;
                    s2 = __builtin_fmaf(d, d, s2);
                }
            }
            s1 = wide_block_sum<THREADS>(s1, red);
            s2 = wide_block_sum<THREADS>(s2, red);
            dm = s1 * inv_cols;
            const float var = __builtin_fmaxf(__builtin_fmaf(-dm, dm, s2 * inv_cols), 0.f);
            scale = 1.0f / __builtin_sqrtf(var + eps);
            if (tid == 0) {
                if (stat0) stat0[r] = mean0 + dm;
                if (stat1) stat1[r] = scale;
            }
        }
        YT *yr = y + r * ldy;
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            const int c = j * THREADS + tid;
            if (c < nch) {
                float g[E], o[E];
                load_params<PT, E>(gamma, (int64_t)c * E, g);
                if constexpr (RMS) {
#pragma unroll
                    for (int e = 0; e < E; ++e) o[e] = v[j][e] * scale * g[e];
                } else {
                    float b[E];
                    load_params<PT, E>(beta, (int64_t)c * E, b);
#pragma unroll
                    for (int e = 0; e < E; ++e) o[e] = __builtin_fmaf((v[j][e] - dm) * scale, g[e], b[e]);
                }
                store_chunk<YT, E>(yr + (int64_t)c * E, o);
            }
            __builtin_amdgcn_sched_barrier(0);  // keeps the parameter loads chunk by chunk (register count)
        }
    }
}

// Launch: rows of up to 128 KiB in a workgroup's registers (4 waves up to 32 KiB, 16 beyond); longer
// ones parked in LDS: 16 waves per row beyond 32 KiB of input, else 4; as many workgroups per CU
// as LDS and wave slots allow.  waves_per_row (4 or 16) and grid (workgroups), when not 0, are the
// caller's choice among the register kernels.
// Returns 0 = launched, 1 = the attribute call failed, 2 = the chosen kernel cannot run the rows.
template <typename XT, typename PT, typename YT, bool RMS>
static int launch_norm_wide(const void *x, const void *gamma, const void *beta, void *y, float *stat0, float *stat1,
                            int64_t rows, int64_t cols, int64_t ldx, int64_t ldy, float eps, hipStream_t st,
                            int waves_per_row = 0, int64_t grid = 0)
{
    constexpr int E = Elem<XT>::kPerChunk;
    const int64_t nch = cols / E;
    // (bf16 rows unpack to twice the registers: 8 chunks per thread of a 16-wave workgroup would spill)
    constexpr int64_t kMax16 = (E == 8 ? 4 : 8) * 1024;
    if (waves_per_row == 0 && nch <= kMax16) waves_per_row = nch <= 8 * 256 ? 4 : 16;
    if (waves_per_row != 0) {
        auto reg = [&](auto kern, int threads) {
            (void)threads;
            int64_t blocks = rows < 256 * 16 ? rows : 256 * 16;  // 16 workgroups per CU, as for the softmax
            if (grid > 0) blocks = grid < rows ? grid : rows;
            hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), 0, st, (const XT *)x, (const PT *)gamma,
                               (const PT *)beta, (YT *)y, stat0, stat1, rows, (int)cols, ldx, ldy, eps);
            return 0;
        };
        if (waves_per_row == 4 && nch <= 8 * 256) return reg(norm_wgrow_kernel<XT, PT, YT, 256, 8, RMS>, 256);
        if (waves_per_row == 16 && nch <= 4 * 1024) return reg(norm_wgrow_kernel<XT, PT, YT, 1024, 4, RMS>, 1024);
        if constexpr (E == 4)
            if (waves_per_row == 16 && nch <= 8 * 1024) return reg(norm_wgrow_kernel<XT, PT, YT, 1024, 8, RMS>, 1024);
        return 2;
    }
    const int64_t cap = nch * 16 > kWideRowLdsBytes ? kWideRowLdsBytes / 16 : nch;
    const size_t lds = (size_t)cap * 16;
    auto go = [&](auto kern, int threads) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)kWideRowLdsBytes) != hipSuccess)
            return 1;
        int64_t per_cu = (160 * 1024) / (int64_t)(lds + 256);
        const int64_t by_waves = 2048 / threads;
        per_cu = per_cu < 1 ? 1 : per_cu > by_waves ? by_waves : per_cu;
        const int64_t blocks = rows < 256 * per_cu ? rows : 256 * per_cu;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds, st, (const XT *)x, (const PT *)gamma,
                           (const PT *)beta, (YT *)y, stat0, stat1, rows, cols, ldx, ldy, eps, cap);
        return 0;
    };
    if (nch * 16 > 32 * 1024) return go(norm_wide_kernel<XT, PT, YT, 1024, RMS>, 1024);
    return go(norm_wide_kernel<XT, PT, YT, 256, RMS>, 256);
}

}  // namespace perf
