// Attention-score GEMM with the row softmax as its epilogue, for gfx950:
//     P_b = softmax_rows(alpha * A_b * B_b^T)
// (the "bmm" and "softmax" rows of the operator table, Section 4.3 of the paper, joined the
// way the paper's fusion moves join producer and consumer scopes, Sections 2.2 and 3.1: the
// score matrix never goes to memory, so the traffic is the operands plus one write of P).
//
//  * gemm_softmax_kernel: bf16 operands, both K-contiguous, N <= 512, K = 64 or 128.  A
//    workgroup of 4 waves owns 64 rows x all N columns of one matrix; each wave 16 rows x N
//    as up to 32 accumulators of 16x16 (128 registers), computed with B as the MFMA's row
//    operand, so that a lane holds 4 consecutive columns per accumulator and all of a
//    lane's values belong to ONE row: the row reductions are in-lane plus two lane
//    exchanges, and the write-out is 16 bytes per lane in whole 128-byte segments.  The
//    operand strips and all of B go to LDS (global->LDS loads, the swizzled 128-byte rows
//    of mfma_tile.h): B once per workgroup, which then walks over several row strips of the
//    matrix with the next strip's rows in flight.  With K = 64 two workgroups fit a CU
//    (80 KiB of LDS, <= 256 registers), so one's exponentials overlap the other's stores.
//  * any other legal case: perf_gemm into P followed by perf_softmax in place.
#include <atomic>
#include "mfma_tile.h"
#include "softmax_math.h"
#include "host_utils.h"

namespace perf {

// T16N: 16-column accumulators per wave (N <= 16 * T16N); MASK: N < 16 * T16N.
// A workgroup takes `group` consecutive row strips of one matrix: B goes to LDS once per
// workgroup, and a wave's 16 rows of the next strip are fetched (into the other of two
// buffers; the rows are the wave's own, so no barrier is involved) while it works on the
// present one, so its stores follow each other without a load latency in between.
template <int T16N, bool MASK, typename PT>
__global__ __launch_bounds__(256, 2) void gemm_softmax_kernel(const uint16_t *__restrict__ A,
                                                              const uint16_t *__restrict__ B, PT *__restrict__ P,
                                                              int M, int N, int K, int64_t lda, int64_t ldb,
                                                              int64_t ldp, int64_t strideA, int64_t strideB,
                                                              int64_t strideP, float sign, float c, int strips,
                                                              int group, int xcd_remap)
{
    constexpr int NW = 4, BM = 64, BN = 16 * T16N;
    constexpr int LB = (BN + 8 * NW - 1) / (8 * NW);     // wave loads per K-step of 64 for B (the last one may be partly unused)
    constexpr int kRowsB = LB * 8 * NW;
    constexpr int kStepB = kRowsB * kRowBytes64, kStepA = BM * kRowBytes64;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: LDS addresses stay scalar
    // Workgroup id -> (strip group, matrix).  Ids are dealt round-robin to the 8 XCDs, each with
    // a private L2; with the remap all groups of one matrix run on one XCD, so B is fetched
    // over the fabric once per matrix.
    const int groups = (strips + group - 1) / group;
    int gi, bz;
    if (xcd_remap) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        gi = j % groups;
        bz = (j / groups) * 8 + xcd;
    } else {
        gi = blockIdx.x % groups;
        bz = blockIdx.x / groups;
    }
    const int s0 = gi * group, s1 = min(strips, s0 + group);
    const int ksteps = K / 64;
    const uint16_t *Ab = A + (int64_t)bz * strideA;
    const uint16_t *Bb = B + (int64_t)bz * strideB;
    PT *Pb = P + (int64_t)bz * strideP;
    char *const smem_a = smem + ksteps * kStepB;  // two buffers of ksteps x 64 rows

    // this wave's 16 rows of strip s -> buffer s & 1 (nothing if the rows lie past M)
    auto issue_a = [&](int s) {
        const int row0 = s * BM + wave * 16;
        if (row0 >= M) return;
        RowMajorSrc64<2, 1> src(Ab + (int64_t)row0 * lda, min(16, M - row0), lda, ksteps, 0, lane);
        char *buf = smem_a + (s & 1) * ksteps * kStepA + wave * 16 * kRowBytes64;
        for (int ks = 0; ks < ksteps; ++ks) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t vo = src.voff[i], so = src.soff;
                issue_load_to(src.rsrc, vo, so, buf + ks * kStepA + i * 8 * kRowBytes64);
            }
            src.advance();
        }
    };

    {
        RowMajorSrc64<LB, NW> src_b(Bb, min(kRowsB, N), ldb, ksteps, wave, lane);
        for (int ks = 0; ks < ksteps; ++ks) {
#pragma unroll
            for (int i = 0; i < LB; ++i) {
                const uint32_t vo = src_b.voff[i], so = src_b.soff;
                issue_load_to(src_b.rsrc, vo, so, smem + ks * kStepB + (i * NW + wave) * 8 * kRowBytes64);
            }
            src_b.advance();
        }
    }
    issue_a(s0);
    wait_vmem<0>();
    wg_barrier();  // B is complete (and each wave's own rows of the first strip)

    for (int s = s0; s < s1; ++s) {
        if (s + 1 < s1) issue_a(s + 1);  // (they have landed before this strip's stores are issued, see below)
        const int m0 = s * BM;
        if (m0 + wave * 16 >= M) continue;  // (no barrier inside the loop)
        const char *abuf = smem_a + (s & 1) * ksteps * kStepA;

        // acc[j] element e: row m0 + 16*wave + lane%16, column 16 j + 4 (lane/16) + e
        WaveTile16<1, T16N> t;
        t.clear();
        for (int ks = 0; ks < ksteps; ++ks) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int chunk = 4 * half + (lane >> 4);
                const bf16x8_t a =
                    *reinterpret_cast<const bf16x8_t *>(abuf + ks * kStepA + frag_offset64(wave * 16 + (lane & 15), chunk));
#pragma unroll
                for (int j = 0; j < T16N; ++j) {
                    const bf16x8_t b = *reinterpret_cast<const bf16x8_t *>(smem + ks * kStepB +
                                                                            frag_offset64(j * 16 + (lane & 15), chunk));
                    t.acc[0][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b, a, t.acc[0][j], 0, 0, 0);
                }
            }
        }
        // the reads of this strip's rows are back before the buffer is refilled two strips on
        // (the compiler waits for them in front of the MFMAs that use them)

        // Row softmax.  All of a lane's values belong to row lane%16; lanes l, l^16, l^32, l^48
        // share it.  exp(|alpha| * (v - m)) is evaluated as exp2 of a plain product: its relative
        // error is ~2^-24 times the exponent, i.e. below 4e-6 for every result above 2^-100, and
        // smaller results are below the floor under which only the absolute error is specified.
        float m = -FLT_MAX;
#pragma unroll
        for (int j = 0; j < T16N; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v = t.acc[0][j][e] * sign;
                if (MASK) v = (16 * j + 4 * (lane >> 4) + e < N) ? v : -FLT_MAX;
                t.acc[0][j][e] = v;
                m = __builtin_fmaxf(m, v);
            }
        {
            float a, b;
            swap16(m, a, b);
            m = __builtin_fmaxf(a, b);
            swap32(m, a, b);
            m = __builtin_fmaxf(a, b);
        }
        float z = 0.f;
#pragma unroll
        for (int j = 0; j < T16N; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float p = __builtin_amdgcn_exp2f((t.acc[0][j][e] - m) * c);
                if (MASK) p = (16 * j + 4 * (lane >> 4) + e < N) ? p : 0.f;  // (c == 0 would give masked columns weight 1)
                t.acc[0][j][e] = p;
                z += p;
            }
        {
            float a, b;
            swap16(z, a, b);
            z = a + b;
            swap32(z, a, b);
            z = a + b;
        }
        // The next strip's rows must have landed before they are read: waiting here, where those
        // loads are a whole strip's arithmetic old, costs least.  It also waits for the previous
        // strip's stores, i.e. a wave has one strip of stores in flight (32 KiB; 256 KiB per CU),
        // which is more than the write latency needs.
        wait_vmem<0>();
        store_tile16<1, T16N, PT>(t, Pb, ldp, M, N, m0 + wave * 16, 0, 1.0f / z, lane);
    }
}

template <int T16N, bool MASK, typename PT>
static perf_status launch_fused(const void *A, const void *B, void *P, int64_t M, int64_t N, int64_t K, int64_t lda,
                                int64_t ldb, int64_t ldp, int64_t batch, int64_t strideA, int64_t strideB,
                                int64_t strideP, float alpha, hipStream_t st)
{
    constexpr int kRowsB = (16 * T16N + 31) / 32 * 32;
    const size_t lds = (size_t)(K / 64) * (2 * 64 + kRowsB) * kRowBytes64;  // B, and two buffers for the row strips
    auto kern = gemm_softmax_kernel<T16N, MASK, PT>;
    // the dynamic-LDS cap is a per-function setting: raised once to the CU's 160 KiB (idempotent, so
    // concurrent first calls are harmless)
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                160 * 1024) != hipSuccess)
            return PERF_ERR_LAUNCH;
        attr_done = true;
    }
    const float sign = alpha < 0.f ? -1.f : 1.f;
    const float c = (float)(std::fabs((double)alpha) * 1.4426950408889634074);  // |alpha| log2(e)
    const int64_t strips = (M + 63) / 64;
    // strips per workgroup: as many as still leave two workgroups for every CU
    int64_t group = strips * batch / 512;
    group = group < 1 ? 1 : group > strips ? strips : group;
    const int64_t groups = (strips + group - 1) / group;
    // one-dimensional grid of strip groups x matrices, in chunks that keep the grid below its limit
    const int64_t per_launch = (kMaxGridX / groups) / 8 * 8;
    if (per_launch < 8) return PERF_ERR_UNSUPPORTED;
    for (int64_t b0 = 0; b0 < batch; b0 += per_launch) {
        const int64_t nb = batch - b0 < per_launch ? batch - b0 : per_launch;
        hipLaunchKernelGGL(kern, dim3((unsigned)(groups * nb)), dim3(256), lds, st, (const uint16_t *)A + b0 * strideA,
                           (const uint16_t *)B + b0 * strideB, (PT *)P + b0 * strideP, (int)M, (int)N, (int)K, lda, ldb,
                           ldp, strideA, strideB, strideP, sign, c, (int)strips, (int)group, nb % 8 == 0 ? 1 : 0);
    }
    return launch_status();
}

}  // namespace perf

extern "C" perf_status perf_gemm_softmax(const void *A, const void *B, void *P, int64_t M, int64_t N, int64_t K,
                                         int64_t lda, int64_t ldb, int64_t ldp, int64_t batch, int64_t strideA,
                                         int64_t strideB, int64_t strideP, float alpha, perf_dtype ab_dt,
                                         perf_dtype p_dt, perf_stream stream)
{
    using namespace perf;
    if (!A || !B || !P) return PERF_ERR_NULL;
    if (!dtype_ok(ab_dt) || !dtype_ok(p_dt)) return PERF_ERR_DTYPE;
    if (M < 1 || N < 1 || K < 1 || batch < 1) return PERF_ERR_SHAPE;
    if (lda < K || ldb < K || ldp < N) return PERF_ERR_SHAPE;
    if (strideA < 0 || strideB < 0 || strideP < 0 || !std::isfinite(alpha)) return PERF_ERR_SHAPE;
    if (batch > 1 && strideP < (M - 1) * ldp + N) return PERF_ERR_SHAPE;
    const int64_t kLim = INT64_MAX / 8;
    if (M > kLim / lda || N > kLim / ldb || M > kLim / ldp) return PERF_ERR_SHAPE;
    if (batch > 1 && (strideA > kLim / batch || strideB > kLim / batch || strideP > kLim / batch)) return PERF_ERR_SHAPE;
    if (!aligned(A, dtype_size(ab_dt)) || !aligned(B, dtype_size(ab_dt)) || !aligned(P, dtype_size(p_dt)))
        return PERF_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);

    const bool fused = ab_dt == PERF_BF16 && (K == 64 || K == 128) && N <= 512 && lda % 8 == 0 && ldb % 8 == 0 &&
                       strideA % 8 == 0 && strideB % 8 == 0 && aligned(A, 16) && aligned(B, 16) && lda <= (1 << 21) &&
                       ldb <= (1 << 21) && M <= (1 << 24);
    if (fused) {
#define PERF_FUSED(T, MASK)                                                                                              \
    (p_dt == PERF_F32                                                                                                    \
         ? launch_fused<T, MASK, float>(A, B, P, M, N, K, lda, ldb, ldp, batch, strideA, strideB, strideP, alpha, st)    \
         : launch_fused<T, MASK, uint16_t>(A, B, P, M, N, K, lda, ldb, ldp, batch, strideA, strideB, strideP, alpha, st))
        if (N == 512) return PERF_FUSED(32, false);
        if (N > 256) return PERF_FUSED(32, true);
        if (N == 256) return PERF_FUSED(16, false);
        if (N > 128) return PERF_FUSED(16, true);
        if (N == 128) return PERF_FUSED(8, false);
        if (N > 64) return PERF_FUSED(8, true);
        return PERF_FUSED(4, true);
#undef PERF_FUSED
    }
    // Unfused: scores into P, then the row softmax in place (fp32 P only).
    if (p_dt != PERF_F32) return PERF_ERR_UNSUPPORTED;
    perf_status s = perf_gemm(A, B, P, M, N, K, PERF_ROW_MAJOR, lda, PERF_COL_MAJOR, ldb, ldp, batch, strideA, strideB,
                              strideP, alpha, ab_dt, PERF_F32, stream);
    if (s != PERF_OK) return s;
    if (batch == 1 || strideP == M * ldp) return perf_softmax(P, P, batch * M, N, ldp, ldp, PERF_F32, PERF_F32, 1.0f, stream);
    for (int64_t b = 0; b < batch; ++b) {
        s = perf_softmax((float *)P + b * strideP, (float *)P + b * strideP, M, N, ldp, ldp, PERF_F32, PERF_F32, 1.0f, stream);
        if (s != PERF_OK) return s;
    }
    return PERF_OK;
}
