// Batch normalisation with batch statistics for gfx950 ("batchnorm" rows of the operator
// table, Section 4.3 of the paper; its MI300A case study is this operator: the statistics
// are computed first, then a streaming kernel normalises).  x is NCHW; a channel's data are
// N planes of H*W contiguous elements.
//
//  * bn_partial_kernel: a workgroup reduces one segment (<= 16384 elements) of one plane,
//    held in registers: provisional mean, then first and second moments of the shifted data
//    (the corrected two-pass form of the LayerNorm kernel), written as (mean_hi, mean_lo, M2).
//  * bn_finalize_kernel: one workgroup per channel merges the segments' (count, mean, M2) in
//    double precision (the pairwise update of parallel variance algorithms), and writes mean,
//    rstd and the per-channel scale rstd*gamma.
//  * bn_apply_kernel: streaming y = (x - mean) * scale + beta, 16-byte accesses.
// The partials live in a caller-supplied workspace (perf_batchnorm_workspace_bytes): no
// atomics, results bit-identical from run to run.
#include <atomic>
#include "row_io.h"
#include "host_utils.h"

namespace perf {

constexpr int kBnSeg = 16384;  // elements per segment: 256 threads x 64

__device__ __forceinline__ float bn_block_sum(float v, float *red)
{
    v = wave_allreduce(v, OpSum{});
    __syncthreads();  // red may still be read from the previous use
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// grid: (segments per plane, N*C planes).  VEC: plane size and base allow 16-byte loads.
template <typename XT, bool VEC>
__global__ __launch_bounds__(256) void bn_partial_kernel(const XT *__restrict__ x, float *__restrict__ partial, int64_t HW,
                                                         int C, int segs)
{
    constexpr int E = Elem<XT>::kPerChunk;
    constexpr int kPerThread = kBnSeg / 256;  // 64
    __shared__ float red[4];
    const int64_t plane = blockIdx.y;  // n*C + c
    const int64_t seg0 = (int64_t)blockIdx.x * kBnSeg;
    const bool full = blockIdx.x + 1 < gridDim.x || HW % kBnSeg == 0;  // every segment but a ragged last one
    const int64_t len = full ? (int64_t)kBnSeg : HW - seg0;
    const XT *xp = x + plane * HW + seg0;
    float v[kPerThread];
    if (VEC && full) {
        // full segment (uniform): straight-line loads, all in flight together; with a bounds
        // test around each load the compiler waits for the loads two at a time
#pragma unroll
        for (int j = 0; j < kPerThread / E; ++j)
            Elem<XT>::unpack(*reinterpret_cast<const uint4_t *>(xp + ((int64_t)j * 256 + threadIdx.x) * E), v + j * E);
    } else if (VEC) {
#pragma unroll
        for (int j = 0; j < kPerThread / E; ++j) {
            const int64_t e0 = ((int64_t)j * 256 + threadIdx.x) * E;
            if (e0 < len) {  // HW is a multiple of E: a chunk is entirely inside or outside
                // plain (cacheable) load: what the last-level cache keeps of x is read from there by the
                // apply kernel (8x64x300x300 fp32: 107 -> 89 us)
                Elem<XT>::unpack(*reinterpret_cast<const uint4_t *>(xp + e0), v + j * E);
            } else {
#pragma unroll
                for (int e = 0; e < E; ++e) v[j * E + e] = 0.f;
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < kPerThread; ++j) {
            const int64_t e0 = (int64_t)j * 256 + threadIdx.x;
            v[j] = e0 < len ? Elem<XT>::load1(xp + e0) : 0.f;
        }
    }
    auto inside = [&](int j) {  // is register j a real element?
        const int64_t e0 = VEC ? ((int64_t)(j / E) * 256 + threadIdx.x) * E + j % E : (int64_t)j * 256 + threadIdx.x;
        return e0 < len;
    };
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) s += v[j];  // padding registers hold zeros
    const float inv = 1.0f / (float)len;
    const float mean0 = bn_block_sum(s, red) * inv;
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
        const float d = inside(j) ? v[j] - mean0 : 0.f;
        s1 += d;
        s2 = __builtin_fmaf(d, d, s2);
    }
    s1 = bn_block_sum(s1, red);
    s2 = bn_block_sum(s2, red);
    if (threadIdx.x == 0) {
        const float dm = s1 * inv;
        // segment statistics: mean = mean0 + dm (kept as two floats), M2 = sum (x - mean)^2
        const int c = (int)(plane % C);
        const int64_t n = plane / C;
        float *p = partial + (((int64_t)c * gridDim.y / C + n) * segs + blockIdx.x) * 3;
        p[0] = mean0;
        p[1] = dm;
        p[2] = __builtin_fmaxf(__builtin_fmaf(-dm * (float)len, dm, s2), 0.f);
    }
}

// grid: C workgroups.  coef[c] = rstd*gamma, coef[C + c] = mean.
template <typename PT>
__global__ __launch_bounds__(256) void bn_finalize_kernel(const float *__restrict__ partial, const PT *__restrict__ gamma,
                                                          float *__restrict__ coef, float *__restrict__ mean_out,
                                                          float *__restrict__ rstd_out, int64_t HW, int C, int N, int segs,
                                                          float eps)
{
    __shared__ double sh_n[256], sh_mean[256], sh_m2[256];
    const int c = blockIdx.x;
    const int64_t total = (int64_t)N * segs;
    const float *p = partial + (int64_t)c * total * 3;
    // each thread folds its share of the segments in order, then a tree over the threads
    double cnt = 0.0, mean = 0.0, m2 = 0.0;
    for (int64_t i = threadIdx.x; i < total; i += 256) {
        const int64_t sidx = i % segs;
        const double nb = (double)min((int64_t)kBnSeg, HW - sidx * kBnSeg);
        const double mb = (double)p[3 * i] + (double)p[3 * i + 1], qb = (double)p[3 * i + 2];
        const double nn = cnt + nb, delta = mb - mean;
        mean += delta * (nb / nn);
        m2 += qb + delta * delta * (cnt * nb / nn);
        cnt = nn;
    }
    sh_n[threadIdx.x] = cnt;
    sh_mean[threadIdx.x] = mean;
    sh_m2[threadIdx.x] = m2;
    __syncthreads();
    for (int step = 128; step > 0; step >>= 1) {
        if (threadIdx.x < step) {
            const double na = sh_n[threadIdx.x], nb = sh_n[threadIdx.x + step];
            if (nb > 0.0) {
                const double nn = na + nb, delta = sh_mean[threadIdx.x + step] - sh_mean[threadIdx.x];
                sh_mean[threadIdx.x] += delta * (nb / nn);
                sh_m2[threadIdx.x] += sh_m2[threadIdx.x + step] + delta * delta * (na * nb / nn);
                sh_n[threadIdx.x] = nn;
            }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double var = sh_m2[0] / sh_n[0];
        const float mu = (float)sh_mean[0];
        const float rstd = (float)(1.0 / sqrt(var + (double)eps));
        coef[c] = rstd * Elem<PT>::load1(gamma + c);
        coef[C + c] = mu;
        if (mean_out) mean_out[c] = mu;
        if (rstd_out) rstd_out[c] = rstd;
    }
}

// grid: (segments per plane, N*C planes).
template <typename XT, typename PT, typename YT, bool VEC>
__global__ __launch_bounds__(256) void bn_apply_kernel(const XT *__restrict__ x, const PT *__restrict__ beta,
                                                       const float *__restrict__ coef, YT *__restrict__ y, int64_t HW, int C)
{
    constexpr int E = Elem<XT>::kPerChunk;
    constexpr int kPerThread = kBnSeg / 256;
    const int64_t plane = blockIdx.y;
    const int c = (int)(plane % C);
    const float scale = coef[c], mu = coef[C + c], b = Elem<PT>::load1(beta + c);
    const int64_t seg0 = (int64_t)blockIdx.x * kBnSeg;
    const bool full = blockIdx.x + 1 < gridDim.x || HW % kBnSeg == 0;  // every segment but a ragged last one
    const int64_t len = full ? (int64_t)kBnSeg : HW - seg0;
    const XT *xp = x + plane * HW + seg0;
    YT *yp = y + plane * HW + seg0;
    if (VEC && full) {
        // full segment (uniform): straight-line code; with bounds tests the compiler puts a full
        // wait in front of every store, so each store waits for the one before it
        uint4_t raw[kPerThread / E];
#pragma unroll
        for (int j = 0; j < kPerThread / E; ++j)
            raw[j] = __builtin_nontemporal_load(reinterpret_cast<const uint4_t *>(xp + ((int64_t)j * 256 + threadIdx.x) * E));
#pragma unroll
        for (int j = 0; j < kPerThread / E; ++j) {
            float v[E], o[E];
            Elem<XT>::unpack(raw[j], v);
#pragma unroll
            for (int e = 0; e < E; ++e) o[e] = __builtin_fmaf(v[e] - mu, scale, b);
            store_chunk<YT, E>(yp + ((int64_t)j * 256 + threadIdx.x) * E, o);
        }
    } else if (VEC) {
        uint4_t raw[kPerThread / E];
#pragma unroll
        for (int j = 0; j < kPerThread / E; ++j) {
            const int64_t e0 = ((int64_t)j * 256 + threadIdx.x) * E;
            if (e0 < len) raw[j] = __builtin_nontemporal_load(reinterpret_cast<const uint4_t *>(xp + e0));
        }
#pragma unroll
        for (int j = 0; j < kPerThread / E; ++j) {
            const int64_t e0 = ((int64_t)j * 256 + threadIdx.x) * E;
            if (e0 < len) {
                float v[E], o[E];
                Elem<XT>::unpack(raw[j], v);
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] = __builtin_fmaf(v[e] - mu, scale, b);
                store_chunk<YT, E>(yp + e0, o);
            }
        }
    } else {
        for (int64_t e0 = threadIdx.x; e0 < len; e0 += 256)
            Elem<YT>::store1(yp + e0, __builtin_fmaf(Elem<XT>::load1(xp + e0) - mu, scale, b));
    }
}

struct BnArgs {
    const void *x, *gamma, *beta;
    void *y;
    float *mean_out, *rstd_out, *ws;
    int64_t N, C, HW;
    float eps;
    hipStream_t st;
};

template <typename XT, typename PT, typename YT>
static void launch_bn(const BnArgs &a, bool vec)
{
    const int segs = (int)((a.HW + kBnSeg - 1) / kBnSeg);
    const dim3 grid((unsigned)segs, (unsigned)(a.N * a.C));
    float *partial = a.ws, *coef = a.ws + (int64_t)3 * a.C * a.N * segs;
    if (vec)
        hipLaunchKernelGGL((bn_partial_kernel<XT, true>), grid, dim3(256), 0, a.st, (const XT *)a.x, partial, a.HW,
                           (int)a.C, segs);
    else
        hipLaunchKernelGGL((bn_partial_kernel<XT, false>), grid, dim3(256), 0, a.st, (const XT *)a.x, partial, a.HW,
                           (int)a.C, segs);
    hipLaunchKernelGGL((bn_finalize_kernel<PT>), dim3((unsigned)a.C), dim3(256), 0, a.st, partial, (const PT *)a.gamma,
                       coef, a.mean_out, a.rstd_out, a.HW, (int)a.C, (int)a.N, segs, a.eps);
    if (vec)
        hipLaunchKernelGGL((bn_apply_kernel<XT, PT, YT, true>), grid, dim3(256), 0, a.st, (const XT *)a.x,
                           (const PT *)a.beta, coef, (YT *)a.y, a.HW, (int)a.C);
    else
        hipLaunchKernelGGL((bn_apply_kernel<XT, PT, YT, false>), grid, dim3(256), 0, a.st, (const XT *)a.x,
                           (const PT *)a.beta, coef, (YT *)a.y, a.HW, (int)a.C);
}

template <typename XT, typename PT>
static void launch_bn_y(const BnArgs &a, bool vec, int y_dt)
{
    if (y_dt == PERF_F32) launch_bn<XT, PT, float>(a, vec);
    else launch_bn<XT, PT, uint16_t>(a, vec);
}

static bool bn_shape_ok(int64_t N, int64_t C, int64_t H, int64_t W)
{
    const int64_t kDim = 1 << 24;
    if (N < 1 || C < 1 || H < 1 || W < 1 || N > kDim || C > kDim || H > kDim || W > kDim) return false;
    const int64_t HW = H * W;
    if (N * C > kMaxGridYZ || N * C > (INT64_MAX / 8) / HW) return false;  // planes ride on grid.y
    return true;
}

}  // namespace perf

extern "C" int64_t perf_batchnorm_workspace_bytes(int64_t N, int64_t C, int64_t H, int64_t W)
{
    using namespace perf;
    if (!bn_shape_ok(N, C, H, W)) return -1;
    const int64_t segs = (H * W + kBnSeg - 1) / kBnSeg;
    return 4 * (3 * C * N * segs + 2 * C);
}

namespace perf {

// Scratch of perf_batchnorm_static: the segment partials and the per-channel coefficients that
// perf_batchnorm keeps in the caller's workspace.  One copy per GPU, held until the process ends.
constexpr int64_t kBnStaticFloats = 65536;  // 256 KiB
static __device__ __align__(256) float bn_static_scratch[kBnStaticFloats];

constexpr int kBnMaxDevices = 64;
static std::atomic<float *> bn_static_ptr[kBnMaxDevices];

// Device address of this GPU's copy of the array (the array's name is only a host-side handle).
// Looked up once per device, with that device current; no allocation is involved.
static float *bn_static_address()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kBnMaxDevices) return nullptr;
    float *p = bn_static_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(bn_static_scratch)) != hipSuccess || !sym) return nullptr;
        p = static_cast<float *>(sym);
        bn_static_ptr[dev].store(p, std::memory_order_release);  // every thread computes the same value
    }
    return p;
}

}  // namespace perf

namespace perf {

// Host-side argument checks shared by both entry points (no HIP call).
static perf_status bn_check(const void *x, const void *gamma, const void *beta, const void *y, const float *mean_out,
                            const float *rstd_out, int64_t N, int64_t C, int64_t H, int64_t W, float eps, int x_dt,
                            int param_dt, int y_dt)
{
    if (!x || !gamma || !beta || !y) return PERF_ERR_NULL;
    if (!dtype_ok(x_dt) || !dtype_ok(param_dt) || !dtype_ok(y_dt)) return PERF_ERR_DTYPE;
    if (!bn_shape_ok(N, C, H, W) || !(eps >= 0.f) || !std::isfinite(eps)) return PERF_ERR_SHAPE;
    if (!aligned(x, dtype_size(x_dt)) || !aligned(y, dtype_size(y_dt)) || !aligned(gamma, dtype_size(param_dt)) ||
        !aligned(beta, dtype_size(param_dt)) || (mean_out && !aligned(mean_out, 4)) || (rstd_out && !aligned(rstd_out, 4)))
        return PERF_ERR_ALIGN;
    return PERF_OK;
}

static perf_status bn_run(const void *x, const void *gamma, const void *beta, void *y, float *mean_out, float *rstd_out,
                          float *workspace, int64_t N, int64_t C, int64_t H, int64_t W, float eps, int x_dt, int param_dt,
                          int y_dt, perf_stream stream)
{
    const int64_t HW = H * W, ex = 16 / dtype_size(x_dt);
    // 16-byte path: every plane starts 16-byte aligned in x and y, and holds whole chunks
    const bool vec = HW % ex == 0 && aligned(x, 16) && aligned(y, 16) && (HW * dtype_size(y_dt)) % 16 == 0;
    BnArgs a{x, gamma, beta, y, mean_out, rstd_out, workspace, N, C, HW, eps, static_cast<hipStream_t>(stream)};
    if (x_dt == PERF_F32) {
        if (param_dt == PERF_F32) launch_bn_y<float, float>(a, vec, y_dt);
        else launch_bn_y<float, uint16_t>(a, vec, y_dt);
    } else {
        if (param_dt == PERF_F32) launch_bn_y<uint16_t, float>(a, vec, y_dt);
        else launch_bn_y<uint16_t, uint16_t>(a, vec, y_dt);
    }
    return launch_status();
}

}  // namespace perf

extern "C" perf_status perf_batchnorm(const void *x, const void *gamma, const void *beta, void *y, float *mean_out,
                                      float *rstd_out, void *workspace, int64_t N, int64_t C, int64_t H, int64_t W,
                                      float eps, perf_dtype x_dt, perf_dtype param_dt, perf_dtype y_dt, perf_stream stream)
{
    using namespace perf;
    if (!workspace) return PERF_ERR_NULL;
    const perf_status s = bn_check(x, gamma, beta, y, mean_out, rstd_out, N, C, H, W, eps, x_dt, param_dt, y_dt);
    if (s != PERF_OK) return s;
    if (!aligned(workspace, 4)) return PERF_ERR_ALIGN;
    return bn_run(x, gamma, beta, y, mean_out, rstd_out, static_cast<float *>(workspace), N, C, H, W, eps, x_dt, param_dt,
                  y_dt, stream);
}

extern "C" int64_t perf_batchnorm_static_max_bytes(void) { return 4 * perf::kBnStaticFloats; }

extern "C" perf_status perf_batchnorm_static(const void *x, const void *gamma, const void *beta, void *y,
                                             float *mean_out, float *rstd_out, int64_t N, int64_t C, int64_t H,
                                             int64_t W, float eps, perf_dtype x_dt, perf_dtype param_dt,
                                             perf_dtype y_dt, perf_stream stream)
{
    using namespace perf;
    const perf_status s = bn_check(x, gamma, beta, y, mean_out, rstd_out, N, C, H, W, eps, x_dt, param_dt, y_dt);
    if (s != PERF_OK) return s;
    if (perf_batchnorm_workspace_bytes(N, C, H, W) > perf_batchnorm_static_max_bytes())
        return PERF_ERR_UNSUPPORTED;  // the problem needs more scratch than the built-in array holds
    float *scratch = bn_static_address();  // first HIP call: every check above ran without one
    if (!scratch) return PERF_ERR_LAUNCH;
    return bn_run(x, gamma, beta, y, mean_out, rstd_out, scratch, N, C, H, W, eps, x_dt, param_dt, y_dt, stream);
}
