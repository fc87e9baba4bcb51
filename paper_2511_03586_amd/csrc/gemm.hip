// Dense / batched GEMM for gfx950 ("matmul" and "bmm" rows of the operator table,
// Section 4.3 of the paper):  C_b = alpha * A_b * B_b, fp32 accumulation.
//
//  * gemm_mfma_kernel: bf16 operands, A row-major and B column-major (both K-contiguous),
//    K a multiple of 32.  256x256, 128x128 or 64x64 workgroup tile; the K-step-64 loop of
//    mfma_tile.h when K is a multiple of 64, else its K-step-32 loop.
//  * f32mfma_kernel (f32mfma.h): any layout / dtype / size (fp32 operands, other layouts, odd K):
//    the fp32 matrix instruction on operands staged through LDS as fp32.
#include <atomic>
#include "mfma_tile.h"
#include "f32mfma.h"
#include "host_utils.h"
#include "timeline.h"

namespace perf {

// Workgroup id -> output tile.  Workgroups are dealt round-robin to the 8 XCDs, each
// with a private L2, so ids that share an XCD (equal id mod 8) are given a contiguous
// run of tiles, and runs walk the tile grid in column-major bands of 4 tile-rows: the
// ~32 tiles an XCD works on at once then form a compact patch sharing A and B panels.
__device__ __forceinline__ void tile_of_block(int bid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int total = tiles_m * tiles_n;
    int id = bid;
    if (total % 8 == 0) id = (bid % 8) * (total / 8) + bid / 8;
    constexpr int kBand = 4;
    const int band_tiles = kBand * tiles_n;
    const int band = id / band_tiles;
    const int rows_in_band = min(kBand, tiles_m - band * kBand);
    const int within = id - band * band_tiles;
    tm = band * kBand + within % rows_in_band;
    tn = within / rows_in_band;
}

template <int TM, int TN, int WM, int WN, bool K64, typename CT, int NS = kStages, bool MI32 = false>
__global__ __launch_bounds__(64 * WM * WN) void gemm_mfma_kernel(const uint16_t *__restrict__ A,
                                                                 const uint16_t *__restrict__ B, CT *__restrict__ C,
                                                                 int M, int N, int K, int64_t lda, int64_t ldb,
                                                                 int64_t ldc, int64_t strideA, int64_t strideB,
                                                                 int64_t strideC, float alpha, int tiles_m, int tiles_n)
{
    using Shape = TileShape<TM, TN, WM, WN, NS>;
    constexpr int BM = Shape::BM, BN = Shape::BN, NW = Shape::kWaves;
    static_assert(!K64 || NS == kStages, "the ring depth is a parameter of the K-step-32 loop only");
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: LDS addresses stay scalar
    TL_BEGIN();
    const int wm = wave / WN, wn = wave % WN;
    // Batches of small matrices (fewer than 8 tiles each): workgroups are dealt round-robin to
    // the 8 XCDs in linear grid order, so the tiles of one matrix would land on different
    // XCDs and its operands would cross the fabric once per tile.  Remap so that a matrix
    // stays on one XCD (needs a multiple of 8 matrices in the launch).
    int bid = blockIdx.x, bz = blockIdx.y;
    const int tiles = tiles_m * tiles_n;
    if (tiles < 8 && gridDim.y % 8 == 0) {
        const unsigned id = blockIdx.x + (unsigned)tiles * blockIdx.y;
        const unsigned xcd = id & 7, j = id >> 3;
        bid = (int)(j % (unsigned)tiles);
        bz = (int)((j / (unsigned)tiles) * 8 + xcd);
    }
    int tm, tn;
    tile_of_block(bid, tiles_m, tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int ktiles = K / kBK;

    {
        const uint16_t *Ab = A + (int64_t)bz * strideA;
        const uint16_t *Bb = B + (int64_t)bz * strideB;
        CT *Cb = C + (int64_t)bz * strideC;

        const int a_row0 = wm * 32 * TM, b_row0 = wn * 32 * TN;
        if constexpr (K64 && MI32) {
            RowMajorSrc64<BM / (8 * NW), NW> src_a(Ab + (int64_t)m0 * lda, min(BM, M - m0), lda, K / 64, wave, lane);
            RowMajorSrc64<BN / (8 * NW), NW> src_b(Bb + (int64_t)n0 * ldb, min(BN, N - n0), ldb, K / 64, wave, lane);
            WaveTile<TM, TN> t;
            t.clear();
            mfma_mainloop_k64_mi32<TM, TN, WM, WN>(t, smem, K / 64, wave, lane, a_row0, b_row0, src_a, src_b);
            store_tile<TM, TN, CT>(t, Cb, ldc, M, N, m0 + a_row0, n0 + b_row0, alpha, lane);
        } else if constexpr (K64) {
            RowMajorSrc64<BM / (8 * NW), NW> src_a(Ab + (int64_t)m0 * lda, min(BM, M - m0), lda, K / 64, wave, lane);
            RowMajorSrc64<BN / (8 * NW), NW> src_b(Bb + (int64_t)n0 * ldb, min(BN, N - n0), ldb, K / 64, wave, lane);
            WaveTile16<2 * TM, 2 * TN> t;
            t.clear();
            TL_STAMP(wave == 0, 0, 2);
            mfma_mainloop_k64<TM, TN, WM, WN>(t, smem, K / 64, wave, lane, a_row0, b_row0, src_a, src_b);
            TL_STAMP(wave == 0, 0, 3);
            if constexpr (sizeof(CT) == 2) {
                // bf16 C: through LDS, so that the stores are 16 bytes per lane in whole rows
                wg_barrier();  // every wave has left the main loop and its loads have landed: LDS is free
                constexpr int kWaveStage = (32 * TM) * (64 * TN);
                static_assert(NW * kWaveStage <= Shape::kLdsBytes, "the staged tiles fit the main loop's LDS");
                if (!store_tile16_bf16<2 * TM, 2 * TN>(t, Cb, ldc, M, N, m0 + a_row0, n0 + b_row0, alpha, lane,
                                                      smem + wave * kWaveStage))
                    store_tile16<2 * TM, 2 * TN, CT>(t, Cb, ldc, M, N, m0 + a_row0, n0 + b_row0, alpha, lane);
            } else {
                store_tile16<2 * TM, 2 * TN, CT>(t, Cb, ldc, M, N, m0 + a_row0, n0 + b_row0, alpha, lane);
            }
            TL_STAMP(wave == 0, 0, 4);
            TL_DRAIN();
            TL_END(wave == 0, 0);
        } else {
            RowMajorSrc<Shape::kLoadsA, NW> src_a(Ab + (int64_t)m0 * lda, min(BM, M - m0), lda, ktiles, wave, lane);
            RowMajorSrc<Shape::kLoadsB, NW> src_b(Bb + (int64_t)n0 * ldb, min(BN, N - n0), ldb, ktiles, wave, lane);
            WaveTile<TM, TN> t;
            t.clear();
            mfma_mainloop<TM, TN, WM, WN, NS>(t, smem, ktiles, wave, lane, a_row0, b_row0, src_a, src_b);
            store_tile<TM, TN, CT>(t, Cb, ldc, M, N, m0 + a_row0, n0 + b_row0, alpha, lane);
        }
    }
}

struct GemmArgs {
    const void *A, *B;
    void *C;
    int64_t M, N, K, lda, ldb, ldc, batch, strideA, strideB, strideC;
    int la, lb;
    float alpha;
    hipStream_t st;
};

template <int TM, int TN, int WM, int WN, bool K64, typename CT, int NS = kStages, bool MI32 = false>
static perf_status launch_mfma(const GemmArgs &g)
{
    using Shape = TileShape<TM, TN, WM, WN, NS>;
    constexpr int BM = Shape::BM, BN = Shape::BN;
    const int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (int)((g.N + BN - 1) / BN);
    const size_t lds = Shape::kLdsBytes;
    auto kern = gemm_mfma_kernel<TM, TN, WM, WN, K64, CT, NS, MI32>;
    static std::atomic<bool> attr_done{false};  // raising the dynamic-LDS cap is a per-function, idempotent setting
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return PERF_ERR_LAUNCH;
        attr_done = true;
    }
    // grid.y carries the batch index; batches beyond the grid limit take further launches
    for (int64_t b0 = 0; b0 < g.batch; b0 += kMaxGridYZ) {
        const unsigned gy = (unsigned)(g.batch - b0 < kMaxGridYZ ? g.batch - b0 : kMaxGridYZ);
        hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n), gy), dim3(Shape::kThreads), lds, g.st,
                           (const uint16_t *)g.A + b0 * g.strideA, (const uint16_t *)g.B + b0 * g.strideB,
                           (CT *)g.C + b0 * g.strideC, (int)g.M, (int)g.N, (int)g.K, g.lda, g.ldb, g.ldc, g.strideA,
                           g.strideB, g.strideC, g.alpha, tiles_m, tiles_n);
    }
    return launch_status();
}

template <typename T, typename CT>
static perf_status launch_general(const GemmArgs &g)
{
    const int64_t a_sm = g.la == PERF_ROW_MAJOR ? g.lda : 1, a_sk = g.la == PERF_ROW_MAJOR ? 1 : g.lda;
    const int64_t b_sk = g.lb == PERF_ROW_MAJOR ? g.ldb : 1, b_sn = g.lb == PERF_ROW_MAJOR ? 1 : g.ldb;
    // 128 x 128 tiles when they give every CU a workgroup, else 64 x 64
    const bool big = ((g.M + 127) / 128) * ((g.N + 127) / 128) * g.batch >= 256;
    const int64_t edge = big ? 128 : 64;
    const int64_t gx = (g.M + edge - 1) / edge, gy = (g.N + edge - 1) / edge;
    if (gx > kMaxGridX || gy > kMaxGridYZ) return PERF_ERR_UNSUPPORTED;
    const unsigned gz = (unsigned)(g.batch < kMaxGridYZ ? g.batch : kMaxGridYZ);
    const DenseRows<T> a_src{(const T *)g.A, a_sm, a_sk, g.M, g.K};
    auto kern = big ? f32mfma_kernel<2, 2, DenseRows<T>, T, CT> : f32mfma_kernel<1, 1, DenseRows<T>, T, CT>;
    hipLaunchKernelGGL(kern, dim3((unsigned)gx, (unsigned)gy, gz), dim3(256), 0, g.st, a_src, (const T *)g.B, (CT *)g.C,
                       g.M, g.N, g.K, b_sk, b_sn, g.ldc, g.strideA, g.strideB, g.strideC, g.batch, g.alpha);
    return launch_status();
}

}  // namespace perf

namespace perf {

template <int TM, int TN, int WM, int WN>
static perf_status launch_mfma_rt(const GemmArgs &g, bool k64, bool c_f32)
{
    if (k64) return c_f32 ? launch_mfma<TM, TN, WM, WN, true, float>(g) : launch_mfma<TM, TN, WM, WN, true, uint16_t>(g);
    return c_f32 ? launch_mfma<TM, TN, WM, WN, false, float>(g) : launch_mfma<TM, TN, WM, WN, false, uint16_t>(g);
}

constexpr int kDeepRing = 33;  // `kstep` code of the K-step-32 loop with the deep ring
constexpr int kK64Mi32 = 65;  // `kstep` code of the K-step-64 loop with 32x32x16 MFMAs (256x256 tile)

// tile / kstep: 0 = chosen here from the shape; otherwise the caller's choice (perf_gemm_variant).
static perf_status gemm_impl(const void *A, const void *B, void *C, int64_t M, int64_t N, int64_t K, perf_layout la,
                             int64_t lda, perf_layout lb, int64_t ldb, int64_t ldc, int64_t batch, int64_t strideA,
                             int64_t strideB, int64_t strideC, float alpha, perf_dtype ab_dt, perf_dtype c_dt,
                             perf_stream stream, int tile, int kstep)
{
    // (argument checks first: they run for every variant)
    if (!A || !B || !C) return PERF_ERR_NULL;
    if (!dtype_ok(ab_dt) || !dtype_ok(c_dt)) return PERF_ERR_DTYPE;
    if (!layout_ok(la) || !layout_ok(lb)) return PERF_ERR_LAYOUT;
    if (M < 1 || N < 1 || K < 1 || batch < 1) return PERF_ERR_SHAPE;
    if (lda < (la == PERF_ROW_MAJOR ? K : M) || ldb < (lb == PERF_ROW_MAJOR ? N : K) || ldc < N) return PERF_ERR_SHAPE;
    if (strideA < 0 || strideB < 0 || strideC < 0 || !std::isfinite(alpha)) return PERF_ERR_SHAPE;
    if (batch > 1 && strideC < (M - 1) * ldc + N) return PERF_ERR_SHAPE;
    // extents must be addressable with 63-bit element offsets
    const int64_t kLim = INT64_MAX / 8;
    const int64_t a_rows = la == PERF_ROW_MAJOR ? M : K, b_rows = lb == PERF_ROW_MAJOR ? K : N;
    if (a_rows > kLim / lda || b_rows > kLim / ldb || M > kLim / ldc) return PERF_ERR_SHAPE;
    if (batch > 1 && (strideA > kLim / batch || strideB > kLim / batch || strideC > kLim / batch)) return PERF_ERR_SHAPE;
    if (ab_dt == PERF_F32 && c_dt == PERF_BF16) return PERF_ERR_UNSUPPORTED;
    if (!aligned(A, dtype_size(ab_dt)) || !aligned(B, dtype_size(ab_dt)) || !aligned(C, dtype_size(c_dt)))
        return PERF_ERR_ALIGN;

    GemmArgs g{A, B, C, M, N, K, lda, ldb, ldc, batch, strideA, strideB, strideC, la, lb, alpha,
               static_cast<hipStream_t>(stream)};
    const bool mfma_ok = ab_dt == PERF_BF16 && la == PERF_ROW_MAJOR && lb == PERF_COL_MAJOR && K % kBK == 0 &&
                         lda % 8 == 0 && ldb % 8 == 0 && strideA % 8 == 0 && strideB % 8 == 0 && aligned(A, 16) &&
                         aligned(B, 16) && lda <= (1 << 21) && ldb <= (1 << 21) && M <= (1 << 30) && N <= (1 << 30) && K <= (1 << 30) &&
                         ((M + 63) / 64) * ((N + 63) / 64) <= kMaxGridX;
    if (tile != 0 || kstep != 0) {  // the caller's variant: only the MFMA kernels have variants
        if (!mfma_ok || (tile != 64 && tile != 128 && tile != 256) ||
            (kstep != 32 && kstep != 64 && kstep != kDeepRing && kstep != kK64Mi32) ||
            ((kstep == 64 || kstep == kK64Mi32) && K % 64 != 0) || (kstep == kDeepRing && tile == 256) ||
            (kstep == kK64Mi32 && tile != 256))
            return PERF_ERR_UNSUPPORTED;
    }
    if (mfma_ok) {
        if (tile == 0) {
            // the 256x256 tile needs enough tiles to occupy the 256 CUs; otherwise 128x128, or 64x64
            // when 128x128 tiles would leave most of the CUs idle
            const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256) * batch;
            const int64_t mid_tiles = ((M + 127) / 128) * ((N + 127) / 128) * batch;
            tile = big_tiles >= 256 ? 256 : mid_tiles >= 192 ? 128 : 64;
            // the K-step-64 loop pays off for the 256x256 tile with a long reduction; short
            // reductions are bound by the C store, which the other loop's epilogue (two full
            // 128-byte row segments per store instruction, no lane exchange) does faster (measured
            // on 512 x (512x512x64)), and the smaller tiles measured faster on the K-step-32 loop on
            // every shape tried.  When a single round of 64x64 tiles has a long reduction, the deep
            // ring keeps 15 K-steps in flight (1024x1024x4096: 23.9 -> 20.2 us); it takes all the LDS,
            // so it loses as soon as a CU should hold more than one workgroup.
            const int64_t small_tiles = ((M + 63) / 64) * ((N + 63) / 64) * batch;
            kstep = (tile == 256 && K % 64 == 0 && K >= 512) ? 64
                    : (tile == 64 && small_tiles <= 256 && K >= 2048) ? kDeepRing
                                                                      : 32;
        }
        const bool k64 = kstep == 64, c_f32 = c_dt == PERF_F32;
        if (kstep == kK64Mi32)
            return c_f32 ? launch_mfma<4, 4, 2, 2, true, float, kStages, true>(g)
                         : launch_mfma<4, 4, 2, 2, true, uint16_t, kStages, true>(g);
        if (kstep == kDeepRing) {  // K-step 32, ring as deep as the LDS allows: 128 KiB either way
            if (tile == 128)
                return c_f32 ? launch_mfma<2, 2, 2, 2, false, float, 8>(g) : launch_mfma<2, 2, 2, 2, false, uint16_t, 8>(g);
            return c_f32 ? launch_mfma<1, 1, 2, 2, false, float, 16>(g) : launch_mfma<1, 1, 2, 2, false, uint16_t, 16>(g);
        }
        if (tile == 256) return launch_mfma_rt<4, 4, 2, 2>(g, k64, c_f32);
        if (tile == 128) return launch_mfma_rt<2, 2, 2, 2>(g, k64, c_f32);
        return launch_mfma_rt<1, 1, 2, 2>(g, k64, c_f32);
    }
    if (ab_dt == PERF_BF16)
        return c_dt == PERF_F32 ? launch_general<uint16_t, float>(g) : launch_general<uint16_t, uint16_t>(g);
    return launch_general<float, float>(g);
}

}  // namespace perf

extern "C" perf_status perf_gemm(const void *A, const void *B, void *C, int64_t M, int64_t N, int64_t K,
                                 perf_layout la, int64_t lda, perf_layout lb, int64_t ldb, int64_t ldc, int64_t batch,
                                 int64_t strideA, int64_t strideB, int64_t strideC, float alpha, perf_dtype ab_dt,
                                 perf_dtype c_dt, perf_stream stream)
{
    return perf::gemm_impl(A, B, C, M, N, K, la, lda, lb, ldb, ldc, batch, strideA, strideB, strideC, alpha, ab_dt, c_dt,
                           stream, 0, 0);
}

extern "C" perf_status perf_gemm_variant(const void *A, const void *B, void *C, int64_t M, int64_t N, int64_t K,
                                         perf_layout la, int64_t lda, perf_layout lb, int64_t ldb, int64_t ldc,
                                         int64_t batch, int64_t strideA, int64_t strideB, int64_t strideC, float alpha,
                                         perf_dtype ab_dt, perf_dtype c_dt, int tile, int kstep, perf_stream stream)
{
    if (tile == 0 || kstep == 0) return PERF_ERR_UNSUPPORTED;
    return perf::gemm_impl(A, B, C, M, N, K, la, lda, lb, ldb, ldc, batch, strideA, strideB, strideC, alpha, ab_dt, c_dt,
                           stream, tile, kstep);
}

#ifdef PERF_TIMELINE
// diagnostic build only: the stamps of the last launches of this file's kernels
extern "C" int perf_timeline_fetch_gemm(long long *host_out) { return perf::tl_fetch(host_out); }
#endif
