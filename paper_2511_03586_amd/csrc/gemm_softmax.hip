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
// STAGED (8 waves, one workgroup per CU, K = 64, N a multiple of 128, fp32 P): the probabilities leave through
// a private 8 KiB LDS region per wave, 128 columns at a time, so that a store instruction writes 2 rows x
// 512 contiguous bytes instead of 8 rows x 128.  A write-only probe of this output (a wave writing its 16
// rows of 2 KiB per strip) moves 5.6 TB/s in the first shape and 6.3 in the second (6.4 with 1 KiB per row,
// for which the LDS has no room): the shape of the store instruction, not the exponentials, held the
// kernel at 0.68 of the HBM peak.
template <int T16N, bool MASK, typename PT, int NW = 4, bool STAGED = false>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void gemm_softmax_kernel(const uint16_t *__restrict__ A,
                                                              const uint16_t *__restrict__ B, PT *__restrict__ P,
                                                              int M, int N, int K, int64_t lda, int64_t ldb,
                                                              int64_t ldp, int64_t strideA, int64_t strideB,
                                                              int64_t strideP, float sign, float c, int strips,
                                                              int group, int xcd_remap)
{
    constexpr int BM = 16 * NW, BN = 16 * T16N;
    static_assert(!STAGED || (!MASK && T16N % 8 == 0 && sizeof(PT) == 4), "the staged write-out takes whole chunks of 128 fp32 columns");
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
    char *const smem_a = smem + ksteps * kStepB;  // two buffers of ksteps x BM rows
    char *const stage = smem_a + 2 * ksteps * kStepA + wave * (16 * 512);  // STAGED: this wave's 16 rows x 128 columns

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
        if (s + 1 < s1) issue_a(s + 1);
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
        const float scale = 1.0f / z;
        // The next strip's rows must have landed before they are read: waiting here, in front of this strip's
        // stores, leaves those in flight across the next strip's MFMAs.  (Letting two strips of stores stay in
        // flight, by waiting for a count at the top of the loop instead, measured no faster.)
        wait_vmem<0>();
        if constexpr (!STAGED) {
            store_tile16<1, T16N, PT>(t, Pb, ldp, M, N, m0 + wave * 16, 0, scale, lane);
        } else {
            // 128 columns at a time: lane (row r = lane % 16, q = lane / 16) writes its 16-byte pieces 4 jj + q of
            // the chunk to row r of the staging; a row is 32 pieces, piece s at position s ^ r (then both the
            // writes, 16 rows per quarter-wave, and the reads, 16 consecutive pieces of a row, are conflict
            // free at a pitch of 512 bytes); then 8 instructions read and store 2 rows x 512 bytes each.
            const int r = lane & 15, q = lane >> 4, piece = lane & 31, half = lane >> 5;
            const int64_t row_base = (int64_t)(m0 + wave * 16);
#pragma unroll
            for (int ch = 0; ch < T16N / 8; ++ch) {
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                    const float4_t v = t.acc[0][8 * ch + jj] * scale;
                    *reinterpret_cast<float4_t *>(stage + r * 512 + (((4 * jj + q) ^ r) << 4)) = v;
                }
                __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): own writes are in LDS (the region is this wave's alone)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int R = 2 * i + half;
                    const float4_t v = *reinterpret_cast<const float4_t *>(stage + R * 512 + ((piece ^ R) << 4));
                    if (row_base + R < M)
                        __builtin_nontemporal_store(v, reinterpret_cast<float4_t *>(Pb + (row_base + R) * ldp + ch * 128 + piece * 4));
                }
            }
        }
    }
}

// The staged form: 8 waves, 128-row strips, 160 KiB of LDS (B 64 KiB, two row buffers of 16 KiB, 64 KiB of staging).
template <int T16N>
static perf_status launch_fused_staged(const void *A, const void *B, void *P, int64_t M, int64_t N, int64_t K, int64_t lda,
                                       int64_t ldb, int64_t ldp, int64_t batch, int64_t strideA, int64_t strideB,
                                       int64_t strideP, float alpha, hipStream_t st)
{
    constexpr int NW = 8;
    constexpr int kRowsB = (16 * T16N + 8 * NW - 1) / (8 * NW) * (8 * NW);
    const size_t lds = (size_t)(K / 64) * (2 * 16 * NW + kRowsB) * kRowBytes64 + (size_t)NW * 16 * 512;
    if (lds > 160 * 1024) return PERF_ERR_UNSUPPORTED;
    auto kern = gemm_softmax_kernel<T16N, false, float, NW, true>;
    static std::atomic<bool> attr_done{false};  // (idempotent per-function setting)
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                160 * 1024) != hipSuccess)
            return PERF_ERR_LAUNCH;
        attr_done = true;
    }
    const float sign = alpha < 0.f ? -1.f : 1.f;
    const float c = (float)(std::fabs((double)alpha) * 1.4426950408889634074);  // |alpha| log2(e)
    const int64_t strips = (M + 16 * NW - 1) / (16 * NW);
    // strips per workgroup: as many as still leave two workgroups for every CU (one runs at a time)
    int64_t group = strips * batch / 512;
    group = group < 1 ? 1 : group > strips ? strips : group;
    const int64_t groups = (strips + group - 1) / group;
    const int64_t per_launch = (kMaxGridX / groups) / 8 * 8;
    if (per_launch < 8) return PERF_ERR_UNSUPPORTED;
    for (int64_t b0 = 0; b0 < batch; b0 += per_launch) {
        const int64_t nb = batch - b0 < per_launch ? batch - b0 : per_launch;
        hipLaunchKernelGGL(kern, dim3((unsigned)(groups * nb)), dim3(64 * NW), lds, st, (const uint16_t *)A + b0 * strideA,
                           (const uint16_t *)B + b0 * strideB, (float *)P + b0 * strideP, (int)M, (int)N, (int)K, lda, ldb,
                           ldp, strideA, strideB, strideP, sign, c, (int)strips, (int)group, nb % 8 == 0 ? 1 : 0);
    }
    return launch_status();
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
        // whole chunks of 128 columns, K = 64, fp32 P with 16-byte aligned rows: the staged write-out
        const bool staged = K == 64 && N % 128 == 0 && p_dt == PERF_F32 && ldp % 4 == 0 && strideP % 4 == 0 && aligned(P, 16);
        if (staged && N == 512) return launch_fused_staged<32>(A, B, P, M, N, K, lda, ldb, ldp, batch, strideA, strideB, strideP, alpha, st);
        if (staged && N == 256) return launch_fused_staged<16>(A, B, P, M, N, K, lda, ldb, ldp, batch, strideA, strideB, strideP, alpha, st);
        if (staged && N == 128) return launch_fused_staged<8>(A, B, P, M, N, K, lda, ldb, ldp, batch, strideA, strideB, strideP, alpha, st);
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
