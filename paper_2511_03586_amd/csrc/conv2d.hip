// 2-D convolution as an implicit GEMM for gfx950 ("conv" rows of the operator table,
// Section 4.3 of the paper; the input index p*stride + r is the paper's
// "expression as location" feature, Section 2.1).
//
// GEMM view: rows m = (n, p, q) output pixels, columns = output channels k, reduction
// index = (r, s, c) with c fastest, which is contiguous in both NHWC activations and KRSC
// weights.  The im2col matrix is never built: for each K-step (one filter tap and one
// 32-channel block) every lane recomputes the byte offset of its 16-byte chunk, and
// taps that fall in the zero padding are given an out-of-range buffer offset, which the
// hardware's buffer range check turns into zeros.
//
//  * conv2d_mfma_kernel: bf16, C a multiple of 32; main loop shared with the GEMM.
//  * conv2d_direct_kernel: any other legal case; one thread per output element.
#include "mfma_tile.h"
#include "host_utils.h"

namespace perf {

struct ConvGeom {
    int N, H, W, C, K, R, S, sh, sw, ph, pw, P, Q;
};

template <int TM, int TN, int WM, int WN, typename CT>
__global__ __launch_bounds__(64 * WM * WN) void conv2d_mfma_kernel(const uint16_t *__restrict__ x,
                                                                   const uint16_t *__restrict__ w, CT *__restrict__ y,
                                                                   ConvGeom g, int tiles_n)
{
    using Shape = TileShape<TM, TN, WM, WN>;
    constexpr int BM = Shape::BM, BN = Shape::BN, NW = Shape::kWaves, LA = Shape::kLoadsA, LB = Shape::kLoadsB;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: LDS addresses stay scalar
    const int wm = wave / WN, wn = wave % WN;
    const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int Mtot = g.N * g.P * g.Q;       // host guarantees this fits in int
    const int cblocks = g.C / kBK;
    const int ktiles = g.R * g.S * cblocks;
    const int64_t ldb = (int64_t)g.R * g.S * g.C;

    // Activations: per load, the pixel this lane fetches for, as the byte offset of its
    // top-left tap (may be negative) and that tap's input coordinates.  Taps in the padding
    // get an out-of-range voffset, which the buffer load turns into zeros.
    struct ActSrc {
        rsrc_t rsrc;
        int64_t pix_off[LA];
        int ih0[LA], iw0[LA];
        int H, W, C, S, cblocks, last;
        __device__ __forceinline__ uint32_t voffset(int kt, int i) const
        {
            kt = min(kt, last);
            const int tap = kt / cblocks, cb = kt % cblocks;
            const int r = tap / S, s = tap % S;
            const int ih = ih0[i] + r, iw = iw0[i] + s;
            const bool inside = ih >= 0 && ih < H && iw >= 0 && iw < W;
            const int64_t off = pix_off[i] + ((int64_t)(r * W + s) * C + cb * kBK) * 2;
            return inside ? (uint32_t)off : kOutOfRange;
        }
        __device__ __forceinline__ uint32_t soffset(int) const { return 0; }
    };
    ActSrc src_a{make_rsrc(x, (uint32_t)((int64_t)g.N * g.H * g.W * g.C * 2)), {}, {}, {}, g.H, g.W, g.C, g.S, cblocks,
                 ktiles - 1};
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int row = load_row<NW>(i, wave, lane);
        const int m = min(m0 + row, Mtot - 1);
        const int n = m / (g.P * g.Q), pq = m % (g.P * g.Q);
        const int p = pq / g.Q, q = pq % g.Q;
        src_a.ih0[i] = p * g.sh - g.ph;
        src_a.iw0[i] = q * g.sw - g.pw;
        src_a.pix_off[i] = (((int64_t)n * g.H + src_a.ih0[i]) * g.W + src_a.iw0[i]) * g.C * 2 + load_chunk(row, lane) * 16;
    }
    const RowMajorSrc<LB, NW> src_b(w + (int64_t)n0 * ldb, min(BN, g.K - n0), ldb, ktiles, wave, lane);

    WaveTile<TM, TN> t;
    t.clear();
    const int a_row0 = wm * 32 * TM, b_row0 = wn * 32 * TN;
    mfma_mainloop<TM, TN, WM, WN>(t, smem, ktiles, wave, lane, a_row0, b_row0, src_a, src_b);
    store_tile<TM, TN, CT>(t, y, g.K, Mtot, g.K, m0 + a_row0, n0 + b_row0, 1.0f, lane);
}

template <typename T> __device__ __forceinline__ float load_xw(const T *p);
template <> __device__ __forceinline__ float load_xw<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float load_xw<uint16_t>(const uint16_t *p) { return bf16_to_f32(*p); }

template <typename T, typename CT>
__global__ __launch_bounds__(256) void conv2d_direct_kernel(const T *__restrict__ x, const T *__restrict__ w,
                                                            CT *__restrict__ y, ConvGeom g, int64_t total)
{
    for (int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (int64_t)gridDim.x * 256) {
        const int k = (int)(o % g.K);
        const int64_t m = o / g.K;
        const int q = (int)(m % g.Q), p = (int)((m / g.Q) % g.P);
        const int64_t n = m / ((int64_t)g.P * g.Q);
        float acc = 0.f;
        for (int r = 0; r < g.R; ++r) {
            const int ih = p * g.sh - g.ph + r;
            if (ih < 0 || ih >= g.H) continue;
            for (int s = 0; s < g.S; ++s) {
                const int iw = q * g.sw - g.pw + s;
                if (iw < 0 || iw >= g.W) continue;
                const T *xp = x + ((n * g.H + ih) * g.W + iw) * g.C;
                const T *wp = w + (((int64_t)k * g.R + r) * g.S + s) * g.C;
                for (int c = 0; c < g.C; ++c) acc = __builtin_fmaf(load_xw<T>(xp + c), load_xw<T>(wp + c), acc);
            }
        }
        store_c<CT>(y + o, acc);
    }
}

template <int TM, int TN, int WM, int WN, typename CT>
static perf_status launch_conv_mfma(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st)
{
    using Shape = TileShape<TM, TN, WM, WN>;
    constexpr int BM = Shape::BM, BN = Shape::BN;
    const int64_t Mtot = (int64_t)g.N * g.P * g.Q;
    const int tiles_m = (int)((Mtot + BM - 1) / BM), tiles_n = (g.K + BN - 1) / BN;
    const size_t lds = Shape::kLdsBytes;
    auto kern = conv2d_mfma_kernel<TM, TN, WM, WN, CT>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return PERF_ERR_LAUNCH;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)((int64_t)tiles_m * tiles_n)), dim3(Shape::kThreads), lds, st,
                       (const uint16_t *)x, (const uint16_t *)w, (CT *)y, g, tiles_n);
    return launch_status();
}

template <typename T, typename CT>
static perf_status launch_conv_direct(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st)
{
    const int64_t total = (int64_t)g.N * g.P * g.Q * g.K;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL((conv2d_direct_kernel<T, CT>), dim3((unsigned)blocks), dim3(256), 0, st, (const T *)x,
                       (const T *)w, (CT *)y, g, total);
    return launch_status();
}

}  // namespace perf

extern "C" perf_status perf_conv2d(const void *x, const void *w, void *y, int64_t N, int64_t H, int64_t W, int64_t C,
                                   int64_t K, int64_t R, int64_t S, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                                   int64_t pad_w, perf_dtype xw_dt, perf_dtype y_dt, perf_stream stream)
{
    using namespace perf;
    if (!x || !w || !y) return PERF_ERR_NULL;
    if (!dtype_ok(xw_dt) || !dtype_ok(y_dt)) return PERF_ERR_DTYPE;
    if (N < 1 || H < 1 || W < 1 || C < 1 || K < 1 || R < 1 || S < 1) return PERF_ERR_SHAPE;
    if (stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0) return PERF_ERR_SHAPE;
    const int64_t kDim = 1 << 24;  // per-dimension cap keeps every product below in 63 bits
    if (N > kDim || H > kDim || W > kDim || C > kDim || K > kDim || R > kDim || S > kDim || stride_h > kDim ||
        stride_w > kDim || pad_h > kDim || pad_w > kDim)
        return PERF_ERR_SHAPE;
    if (H + 2 * pad_h < R || W + 2 * pad_w < S) return PERF_ERR_SHAPE;
    const int64_t P = (H + 2 * pad_h - R) / stride_h + 1, Q = (W + 2 * pad_w - S) / stride_w + 1;
    if (N * P > INT32_MAX / Q) return PERF_ERR_SHAPE;                    // output pixels fit in int
    if (H * W > INT32_MAX / C || R * S > INT32_MAX / C) return PERF_ERR_SHAPE;  // one image / one filter fit in int
    if (N * P * Q > (INT64_MAX / 8) / K || N > (INT64_MAX / 8) / (H * W * C)) return PERF_ERR_SHAPE;
    if (!aligned(x, dtype_size(xw_dt)) || !aligned(w, dtype_size(xw_dt)) || !aligned(y, dtype_size(y_dt)))
        return PERF_ERR_ALIGN;

    ConvGeom g{(int)N, (int)H, (int)W, (int)C, (int)K, (int)R, (int)S, (int)stride_h, (int)stride_w,
               (int)pad_h, (int)pad_w, (int)P, (int)Q};
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool mfma_ok = xw_dt == PERF_BF16 && C % kBK == 0 && aligned(x, 16) && aligned(w, 16) &&
                         N * H * W * C < (int64_t(1) << 30) && K * R * S * C < (int64_t(1) << 30) &&
                         ((N * P * Q + 127) / 128) * ((K + 127) / 128) <= kMaxGridX;
    if (mfma_ok)
        return y_dt == PERF_F32 ? launch_conv_mfma<2, 2, 2, 2, float>(x, w, y, g, st)
                                : launch_conv_mfma<2, 2, 2, 2, uint16_t>(x, w, y, g, st);
    if (xw_dt == PERF_BF16)
        return y_dt == PERF_F32 ? launch_conv_direct<uint16_t, float>(x, w, y, g, st)
                                : launch_conv_direct<uint16_t, uint16_t>(x, w, y, g, st);
    return y_dt == PERF_F32 ? launch_conv_direct<float, float>(x, w, y, g, st)
                            : launch_conv_direct<float, uint16_t>(x, w, y, g, st);
}
