// Contraction on the fp32 matrix instruction for everything the bf16 MFMA kernels do not take:
// fp32 operands, other layouts, odd extents ("matmul", "bmm" and "conv" rows of the operator
// table, Section 4.3 of the paper, which states no data type).
//
//   C[m][n] = alpha * sum_k A(m, k) * B(k, n)
//
// with A given by a row source: a strided matrix (GEMM) or the implicit im2col matrix of a
// convolution (row = output pixel, k = (r, s, c); the paper's expression-as-location indexing,
// Section 2.1), and B a strided matrix.  Operands are staged through LDS as fp32 and multiplied
// with v_mfma_f32_32x32x2_f32.  A workgroup of 2 x 2 waves owns a (64 TM) x (64 TN) tile, a wave
// (32 TM) x (32 TN) of it; two LDS stages; the next K-step's elements are fetched into registers
// while this step's MFMAs run.  Out-of-range elements are zeros, so no extent needs to divide.
// LDS rows are k-major with a pitch of 33 mod 64 floats: the two half-waves of an operand read
// (rows k and k+1, 32 consecutive floats each) overlap in one of the 64 banks only, and the
// transposing write of a K-contiguous operand (consecutive lanes = consecutive k) walks the banks
// with an odd stride instead of hitting two of them (97 -> 50 us on 768x1024x1024).
#pragma once
#include "mfma_tile.h"

namespace perf {

template <typename T> __device__ __forceinline__ float load_ab(const T *p);
template <> __device__ __forceinline__ float load_ab<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float load_ab<uint16_t>(const uint16_t *p) { return bf16_to_f32(*p); }

// Row source: element (m, k) of a strided matrix, A[m*sm + k*sk].
template <typename T>
struct DenseRows {
    const T *p;
    int64_t sm, sk, M, K;
    struct Row {
        int64_t off;
        bool ok;
    };
    __device__ __forceinline__ Row row(int64_t m) const { return Row{min(m, M - 1) * sm, m < M}; }
    __device__ __forceinline__ bool valid(const Row &r, int64_t k) const { return r.ok && k < K; }
    // (clamped, always valid address: the caller zeroes what `valid` rejects)
    __device__ __forceinline__ float load(const Row &r, int64_t k) const { return load_ab<T>(p + r.off + min(k, K - 1) * sk); }
    __device__ __forceinline__ bool k_contiguous() const { return sk == 1; }
    __device__ __forceinline__ void next_matrix(int64_t stride) { p += stride; }
};

// Row source: the implicit im2col matrix of a convolution over NHWC x: row m = output pixel
// (n, p, q), column k = (r, s, c) with c fastest; taps outside the image are zeros.
template <typename T>
struct ConvRows {
    const T *x;
    int H, W, C, S, sh, sw, ph, pw, P, Q;
    int64_t M, K;  // N*P*Q, R*S*C
    struct Row {
        int64_t base;  // element offset of the pixel under tap (0, 0), channel 0 (may lie outside x)
        int ih0, iw0;
        bool ok;
    };
    __device__ __forceinline__ Row row(int64_t m) const
    {
        const int64_t mc = min(m, M - 1);
        const int64_t n = mc / ((int64_t)P * Q);
        const int pq = (int)(mc - n * P * Q), p = pq / Q, q = pq - p * Q;
        const int ih0 = p * sh - ph, iw0 = q * sw - pw;
        return Row{((n * H + ih0) * W + iw0) * C, ih0, iw0, m < M};
    }
    __device__ __forceinline__ void tap(int64_t k, int &r, int &s, int &c) const
    {
        const int kc = (int)min(k, K - 1), t = kc / C;
        c = kc - t * C;
        r = t / S;
        s = t - r * S;
    }
    __device__ __forceinline__ bool valid(const Row &rw, int64_t k) const
    {
        int r, s, c;
        tap(k, r, s, c);
        return rw.ok && k < K && (unsigned)(rw.ih0 + r) < (unsigned)H && (unsigned)(rw.iw0 + s) < (unsigned)W;
    }
    __device__ __forceinline__ float load(const Row &rw, int64_t k) const
    {
        int r, s, c;
        tap(k, r, s, c);
        const bool in = (unsigned)(rw.ih0 + r) < (unsigned)H && (unsigned)(rw.iw0 + s) < (unsigned)W;
        return load_ab<T>(x + (in ? rw.base + ((int64_t)r * W + s) * C + c : 0));  // (element 0 stands in for a padding tap)
    }
    __device__ __forceinline__ bool k_contiguous() const { return true; }
    __device__ __forceinline__ void next_matrix(int64_t) {}
};

template <int TM, int TN, typename ASrc, typename T, typename CT>
__global__ __launch_bounds__(256) void f32mfma_kernel(ASrc a_src, const T *__restrict__ B, CT *__restrict__ C, int64_t M,
                                                      int64_t N, int64_t K, int64_t b_sk, int64_t b_sn, int64_t ldc,
                                                      int64_t strideA, int64_t strideB, int64_t strideC, int64_t batch,
                                                      float alpha)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int BK = TM * TN >= 4 ? 16 : 32;  // (the small tile needs the longer step to cover the fetch latency)
    constexpr int PA = BM + 33, PB = BN + 33;
    constexpr int NA = BM * BK / 256, NB = BN * BK / 256;
    __shared__ float As[2][BK][PA], Bs[2][BK][PB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.x * BM, n0 = (int64_t)blockIdx.y * BN;
    // this thread's elements of a K-step: (row, k) pairs, the contiguous dimension fastest
    int am[NA], ak[NA], bn[NB], bk[NB];
    typename ASrc::Row arow[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int idx = tid + i * 256;
        if (a_src.k_contiguous()) { ak[i] = idx % BK; am[i] = idx / BK; } else { am[i] = idx % BM; ak[i] = idx / BM; }
        arow[i] = a_src.row(m0 + am[i]);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int idx = tid + i * 256;
        if (b_sk == 1) { bk[i] = idx % BK; bn[i] = idx / BK; } else { bn[i] = idx % BN; bk[i] = idx / BN; }
    }
    (void)strideA;
    for (int64_t bz = blockIdx.z; bz < batch; bz += gridDim.z) {
        ASrc a_mat = a_src;
        a_mat.next_matrix(bz * strideA);
        const T *Bb = B + bz * strideB;
        CT *Cb = C + bz * strideC;
        float ra[NA], rb[NB];
        // (loads from clamped, always valid addresses, zeroed when they are parked: a bounds test around
        // each load would make the compiler wait for one load before it issues the next)
        auto fetch = [&](int64_t k0) {
#pragma unroll
            for (int i = 0; i < NA; ++i) ra[i] = a_mat.load(arow[i], k0 + ak[i]);
#pragma unroll
            for (int i = 0; i < NB; ++i)
                rb[i] = load_ab<T>(Bb + min(k0 + bk[i], K - 1) * b_sk + min(n0 + bn[i], N - 1) * b_sn);
        };
        auto park = [&](int buf, int64_t k0) {  // (the first use of the fetched values: the wait for them is here)
#pragma unroll
            for (int i = 0; i < NA; ++i) As[buf][ak[i]][am[i]] = a_mat.valid(arow[i], k0 + ak[i]) ? ra[i] : 0.f;
#pragma unroll
            for (int i = 0; i < NB; ++i) Bs[buf][bk[i]][bn[i]] = (n0 + bn[i] < N && k0 + bk[i] < K) ? rb[i] : 0.f;
        };
        float16_t acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
        fetch(0);
        park(0, 0);
        __syncthreads();
        int buf = 0;
        for (int64_t k0 = 0; k0 < K; k0 += BK) {
            const bool more = k0 + BK < K;
            if (more) fetch(k0 + BK);
#pragma unroll
            for (int kk = 0; kk < BK; kk += 2) {
                float a[TM], b[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) a[i] = As[buf][kk + (lane >> 5)][(wm * TM + i) * 32 + (lane & 31)];
#pragma unroll
                for (int j = 0; j < TN; ++j) b[j] = Bs[buf][kk + (lane >> 5)][(wn * TN + j) * 32 + (lane & 31)];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
            }
            if (more) park(buf ^ 1, k0 + BK);  // (its last readers passed the barrier of the previous step)
            __syncthreads();
            buf ^= 1;
        }
        // accumulator element e: row 8 (e / 4) + 4 (lane / 32) + e % 4, column lane % 32
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int64_t m = m0 + (wm * TM + i) * 32 + 8 * (e / 4) + 4 * (lane >> 5) + e % 4;
                    const int64_t n = n0 + (wn * TN + j) * 32 + (lane & 31);
                    if (m < M && n < N) store_c<CT>(Cb + m * ldc + n, alpha * acc[i][j][e]);
                }
        __syncthreads();  // the stages are refilled for the next matrix
    }
}

}  // namespace perf
