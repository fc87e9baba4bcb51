// Shared bf16 MFMA main loop for gfx950: a workgroup of 4 wavefronts (2 x 2) computes a
// (64*TM) x (64*TN) tile of  sum_k A[m][k] * B[n][k]  with both operands K-contiguous
// ("matmul", "bmm" and "conv" rows of the operator table, Section 4.3 of the paper; the
// tiling / special-instruction / layout moves of Section 2.2 and the independent
// accumulator chains of Section 4.1 are applied by hand here).
//
// Data path per K-step of 64:
//   HBM/L2 --global_load_lds_dwordx4--> LDS (double buffered, XOR-swizzled 16-byte chunks)
//   LDS --ds_read_b128--> operand registers (double buffered per 16-wide k-substep)
//   v_mfma_f32_32x32x16_bf16 into TM*TN independent 32x32 fp32 accumulators per wave.
// One workgroup barrier per K-step, placed before the last k-substep's MFMAs so the first
// operand reads of the next tile overlap with them.
#pragma once
#include "device_utils.h"

namespace perf {

constexpr int kBK = 64;                  // K elements per LDS stage (128 bytes per row)
constexpr int kRowBytes = kBK * 2;
constexpr int kGemmThreads = 256;

// Swizzle: the 16-byte chunk c of tile row r is stored at chunk position c ^ swz(r).
// Rows are 128 bytes, so 16 consecutive rows at a fixed logical chunk land on 16 distinct
// 16-byte slots of a 256-byte bank line (row parity picks the half, (r>>1)&7 the slot).
__device__ __forceinline__ int swz(int r) { return (r >> 1) & 7; }

// s_waitcnt with vmcnt = 0 only (expcnt / lgkmcnt left at "no wait").
__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Issue the direct-to-LDS loads of one ROWS x 64 operand stage.  `src` holds, per load
// issued by this lane, the global address of its 16-byte chunk for the current K-step.
// Load i of wave w fills tile rows (i*4 + w)*8 .. +7: lane l writes row l/8, position l%8.
template <int ROWS>
__device__ __forceinline__ void issue_stage(const char *const (&src)[ROWS / 32], char *lds_stage, int wave)
{
#pragma unroll
    for (int i = 0; i < ROWS / 32; ++i) {
        char *dst = lds_stage + (i * 4 + wave) * 8 * kRowBytes;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src[i],
                                         (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
    }
}

// Byte offset inside a stage of the 16-byte operand fragment a lane feeds to the MFMA:
// tile row `row`, logical chunk `chunk` (= 2*ksub + lane/32).
__device__ __forceinline__ int frag_offset(int row, int chunk)
{
    return row * kRowBytes + ((chunk ^ swz(row)) << 4);
}

template <int TM, int TN>
struct WaveTile {
    float16_t acc[TM][TN];

    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    }
};

template <int TM, int TN>
__device__ __forceinline__ void read_frags(bf16x8_t (&a)[TM], bf16x8_t (&b)[TN], const char *a_stage,
                                           const char *b_stage, int a_row0, int b_row0, int ksub, int lane)
{
    const int chunk = 2 * ksub + (lane >> 5);
#pragma unroll
    for (int i = 0; i < TM; ++i)
        a[i] = *reinterpret_cast<const bf16x8_t *>(a_stage + frag_offset(a_row0 + i * 32 + (lane & 31), chunk));
#pragma unroll
    for (int j = 0; j < TN; ++j)
        b[j] = *reinterpret_cast<const bf16x8_t *>(b_stage + frag_offset(b_row0 + j * 32 + (lane & 31), chunk));
}

template <int TM, int TN>
__device__ __forceinline__ void mma_step(WaveTile<TM, TN> &t, const bf16x8_t (&a)[TM], const bf16x8_t (&b)[TN])
{
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            t.acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], t.acc[i][j], 0, 0, 0);
}

// K loop shared by GEMM and implicit-GEMM convolution.  set_a(kt) / set_b(kt) must leave
// in a_src / b_src the global chunk addresses of K-step kt; they are called once per step,
// in increasing kt, starting at 1 (step 0's addresses are the caller's initial values).
template <int TM, int TN, typename SetA, typename SetB>
__device__ __forceinline__ void mfma_mainloop(WaveTile<TM, TN> &t, const char *(&a_src)[2 * TM],
                                              const char *(&b_src)[2 * TN], char *smem, int ktiles, int wave, int lane,
                                              int a_row0, int b_row0, SetA set_a, SetB set_b)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int kStageBytes = (BM + BN) * kRowBytes;
    bf16x8_t fa[2][TM], fb[2][TN];

    issue_stage<BM>(a_src, smem, wave);
    issue_stage<BN>(b_src, smem + BM * kRowBytes, wave);
    wait_vmem_all();
    __syncthreads();
    read_frags<TM, TN>(fa[0], fb[0], smem, smem + BM * kRowBytes, a_row0, b_row0, 0, lane);

    for (int kt = 0; kt < ktiles; ++kt) {
        char *cur = smem + (kt & 1) * kStageBytes;
        char *nxt = smem + ((kt + 1) & 1) * kStageBytes;
        if (kt + 1 < ktiles) {
            set_a(kt + 1);
            set_b(kt + 1);
            issue_stage<BM>(a_src, nxt, wave);
            issue_stage<BN>(b_src, nxt + BM * kRowBytes, wave);
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int c = ks & 1, n = c ^ 1;
            if (ks < 3) {
                read_frags<TM, TN>(fa[n], fb[n], cur, cur + BM * kRowBytes, a_row0, b_row0, ks + 1, lane);
            } else {
                // the next stage has landed and every wave is done reading the other one
                wait_vmem_all();
                __syncthreads();
                // (after the last K-step this reads stale LDS that is never used)
                read_frags<TM, TN>(fa[n], fb[n], nxt, nxt + BM * kRowBytes, a_row0, b_row0, 0, lane);
            }
            mma_step<TM, TN>(t, fa[c], fb[c]);
        }
    }
}

template <typename CT> __device__ __forceinline__ void store_c(CT *p, float v);
template <> __device__ __forceinline__ void store_c<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_c<uint16_t>(uint16_t *p, float v) { *p = f32_to_bf16(v); }

// Write a wave's accumulators to row-major C.  Accumulator element e of a 32x32 tile is
// row 8*(e/4) + 4*(lane/32) + e%4, column lane%32, so one store instruction writes two
// 128-byte row segments.  (row0, col0) is the wave tile's origin in C.
template <int TM, int TN, typename CT>
__device__ __forceinline__ void store_tile(const WaveTile<TM, TN> &t, CT *C, int64_t ldc, int M, int N, int row0,
                                           int col0, float alpha, int lane)
{
    const int r_l = row0 + 4 * (lane >> 5), c_l = col0 + (lane & 31);
    CT *base = C + (int64_t)r_l * ldc + c_l;
    if (row0 + 32 * TM <= M && col0 + 32 * TN <= N) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                CT *p = base + (int64_t)(i * 32 + 8 * (e >> 2) + (e & 3)) * ldc;
#pragma unroll
                for (int j = 0; j < TN; ++j) store_c<CT>(p + j * 32, alpha * t.acc[i][j][e]);
            }
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int dr = i * 32 + 8 * (e >> 2) + (e & 3);
                CT *p = base + (int64_t)dr * ldc;
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (r_l + dr < M && c_l + j * 32 < N) store_c<CT>(p + j * 32, alpha * t.acc[i][j][e]);
            }
    }
}

}  // namespace perf
