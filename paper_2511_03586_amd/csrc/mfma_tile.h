// Shared bf16 MFMA main loop for gfx950: a workgroup of WM x WN wavefronts, each owning
// TM x TN MFMA tiles of 32x32, computes a (32*TM*WM) x (32*TN*WN) tile of
// sum_k A[m][k] * B[n][k]  with both operands K-contiguous
// ("matmul", "bmm" and "conv" rows of the operator table, Section 4.3 of the paper; the
// tiling / special-instruction / layout moves of Section 2.2 and the independent
// accumulator chains of Section 4.1 are applied by hand here).
//
// Data path per K-step of 32:
//   L2 --buffer_load_dwordx4 ... lds--> LDS ring of 4 stages (XOR-swizzled 16-byte chunks)
//   LDS --ds_read_b128--> operand registers (double buffered per 16-wide k-substep)
//   v_mfma_f32_32x32x16_bf16 into TM*TN independent 32x32 fp32 accumulators per wave.
// Loads run three K-steps ahead of the MFMAs and are issued a few at a time between the
// MFMA groups, so the L2 -> LDS stream is continuous instead of one burst per step; the
// wait before a step's barrier is a partial vmcnt that leaves the two younger steps in
// flight.  One workgroup barrier per K-step, placed before the last k-substep's MFMAs so
// the first operand reads of the next step overlap with them.
#pragma once
#include "device_utils.h"

namespace perf {

constexpr int kBK = 32;                  // K elements per LDS stage (64 bytes per row)
constexpr int kRowBytes = kBK * 2;
constexpr int kStages = 4;

// Swizzle: the 16-byte chunk c (0..3) of tile row r is stored at chunk position c ^ swz(r).
// Rows are 64 bytes, so 16 consecutive rows at one logical chunk land on 16 distinct
// 16-byte slots of the 256-byte LDS bank line: slot = 4*(r%4) + (c ^ (r/4)%4).
__device__ __forceinline__ int swz(int r) { return (r >> 2) & 3; }

// s_waitcnt on vmcnt only (expcnt / lgkmcnt left at "no wait"); gfx9 encoding:
// vmcnt[3:0] in bits 3:0, vmcnt[5:4] in bits 15:14.
template <int N>
__device__ __forceinline__ void wait_vmem()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// Same, and also lgkmcnt = 0 (all of this wave's LDS reads have returned).
template <int N>
__device__ __forceinline__ void wait_vmem_and_lds()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14));
}

// Bare s_barrier: unlike __syncthreads() it carries no fence, so the compiler does not
// drain vmcnt to 0 in front of it; the waits the algorithm needs are written explicitly.
// The empty asm statements stop the compiler from moving memory accesses across it.
__device__ __forceinline__ void wg_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Buffer resource over [base, base + bytes): loads through it take a uniform 32-bit
// soffset and a per-lane 32-bit voffset, so no 64-bit per-lane address arithmetic is
// needed, and a voffset >= bytes reads as zero instead of touching memory.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
constexpr uint32_t kOutOfRange = 0x80000000u;  // voffset of a lane that must read zeros

// One direct-to-LDS load of a wave: 16 tile rows (1 KiB of a stage).  In a workgroup of NW
// waves, load i of wave w fills rows (i*NW + w)*16 .. +15: lane l writes row l/4, chunk
// position l%4.  `wave` must be wave-uniform (an SGPR) so the LDS address is scalar.
template <int NW>
__device__ __forceinline__ void issue_load(rsrc_t rsrc, uint32_t voffset, uint32_t soffset, char *lds_stage, int i,
                                           int wave)
{
    char *dst = lds_stage + (i * NW + wave) * 16 * kRowBytes;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void *)dst, 16, voffset, soffset,
                                             0, 0);
}

// Tile row and swizzled chunk this lane fetches in load i (see issue_load).
template <int NW>
__device__ __forceinline__ int load_row(int i, int wave, int lane) { return (i * NW + wave) * 16 + (lane >> 2); }
__device__ __forceinline__ int load_chunk(int row, int lane) { return (lane & 3) ^ swz(row); }

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

// MFMAs of tile rows [I0, I1) of the wave tile for one 16-wide k-substep.
template <int I0, int I1, int TM, int TN>
__device__ __forceinline__ void mma_rows(WaveTile<TM, TN> &t, const bf16x8_t (&a)[TM], const bf16x8_t (&b)[TN])
{
#pragma unroll
    for (int i = I0; i < I1; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            t.acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], t.acc[i][j], 0, 0, 0);
}

// Geometry of a workgroup tile.
template <int TM, int TN, int WM, int WN>
struct TileShape {
    static constexpr int kWaves = WM * WN;
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    static constexpr int kLoadsA = BM / (16 * kWaves), kLoadsB = BN / (16 * kWaves);  // per lane per K-step
    static constexpr int kStageBytes = (BM + BN) * kRowBytes;
    static constexpr int kLdsBytes = kStages * kStageBytes;
    static_assert(BM % (16 * kWaves) == 0 && BN % (16 * kWaves) == 0, "stage rows must divide among the waves");
};

// Operand stored as rows of K-contiguous bf16 (GEMM A and B, convolution weights): the
// resource starts at the workgroup tile's first row; rows past `rows_valid` re-read the
// last valid row (their products land in outputs that are never stored).
template <int NLOADS, int NW>
struct RowMajorSrc {
    rsrc_t rsrc;
    uint32_t voff[NLOADS];
    int last;

    __device__ __forceinline__ RowMajorSrc(const uint16_t *tile_base, int rows_valid, int64_t ld, int ktiles, int wave,
                                           int lane)
        : rsrc(make_rsrc(tile_base, (uint32_t)(((int64_t)(rows_valid - 1) * ld + (int64_t)ktiles * kBK) * 2))),
          last(ktiles - 1)
    {
#pragma unroll
        for (int i = 0; i < NLOADS; ++i) {
            const int row = load_row<NW>(i, wave, lane);
            voff[i] = (uint32_t)(min(row, rows_valid - 1) * ld * 2) + load_chunk(row, lane) * 16;
        }
    }
    __device__ __forceinline__ uint32_t voffset(int, int i) const { return voff[i]; }
    __device__ __forceinline__ uint32_t soffset(int kt) const { return (uint32_t)min(kt, last) * kRowBytes; }
};

// K loop shared by GEMM and implicit-GEMM convolution.
//   SrcA / SrcB describe where an operand's stage comes from: a buffer resource `rsrc`,
//   voffset(kt, i) = per-lane byte offset of the 16-byte chunk fetched by load i
//   (0 .. kLoadsA-1 / kLoadsB-1) of K-step kt, and soffset(kt) = uniform byte offset of
//   the step.  They are evaluated for kt up to ktiles + 2: steps past the end must still
//   name readable (or out-of-range) bytes; their data lands in a free stage and is never
//   used, which keeps the number of loads in flight, and so the vmcnt waits, uniform.
//   a_row0 / b_row0: first tile row of this wave's operands.  `wave` must be uniform.
template <int TM, int TN, int WM, int WN, typename SrcA, typename SrcB>
__device__ __forceinline__ void mfma_mainloop(WaveTile<TM, TN> &t, char *smem, int ktiles, int wave, int lane,
                                              int a_row0, int b_row0, const SrcA &src_a, const SrcB &src_b)
{
    using Shape = TileShape<TM, TN, WM, WN>;
    constexpr int BM = Shape::BM;
    constexpr int kStageBytes = Shape::kStageBytes;
    constexpr int LA = Shape::kLoadsA, kLoads = Shape::kLoadsA + Shape::kLoadsB;
    static_assert(2 * kLoads < 64, "two K-steps of loads must fit the vmcnt counter");
    bf16x8_t fa[2][TM], fb[2][TN];

    auto issue = [&](int kt, int first, int count) {
        char *stage = smem + (kt % kStages) * kStageBytes;
#pragma unroll
        for (int i = first; i < first + count; ++i) {
            if (i < LA)
                issue_load<Shape::kWaves>(src_a.rsrc, src_a.voffset(kt, i), src_a.soffset(kt), stage, i, wave);
            else
                issue_load<Shape::kWaves>(src_b.rsrc, src_b.voffset(kt, i - LA), src_b.soffset(kt),
                                          stage + BM * kRowBytes, i - LA, wave);
        }
    };

    issue(0, 0, kLoads);
    issue(1, 0, kLoads);
    issue(2, 0, kLoads);
    wait_vmem<2 * kLoads>();  // step 0 has landed
    wg_barrier();
    read_frags<TM, TN>(fa[0], fb[0], smem, smem + BM * kRowBytes, a_row0, b_row0, 0, lane);

    // Each k-substep is ordered by hand with scheduling barriers: the first row of MFMAs
    // goes out, then the operand reads for the next substep, then the remaining MFMAs with
    // the global->LDS loads mixed in.  Reads issued in front of an MFMA group would make the
    // group's own operand wait (an in-order counter) cover them too; reads left to the
    // scheduler sink behind the whole group and their latency is exposed.
    for (int kt = 0; kt < ktiles; ++kt) {
        const char *cur = smem + (kt % kStages) * kStageBytes;
        const char *nxt = smem + ((kt + 1) % kStages) * kStageBytes;
        // k-substep 0
        mma_rows<0, 1>(t, fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        read_frags<TM, TN>(fa[1], fb[1], cur, cur + BM * kRowBytes, a_row0, b_row0, 1, lane);
        __builtin_amdgcn_sched_barrier(0);
        issue(kt + 3, 0, kLoads / 2);
        mma_rows<1, TM>(t, fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        // step kt+1 must have landed (younger loads: step kt+2 and half of kt+3), and every
        // wave must be done reading step kt-1's stage before it is refilled
        wait_vmem_and_lds<kLoads + kLoads / 2>();
        wg_barrier();
        // k-substep 1
        mma_rows<0, 1>(t, fa[1], fb[1]);
        __builtin_amdgcn_sched_barrier(0);
        read_frags<TM, TN>(fa[0], fb[0], nxt, nxt + BM * kRowBytes, a_row0, b_row0, 0, lane);
        __builtin_amdgcn_sched_barrier(0);
        issue(kt + 3, kLoads / 2, kLoads - kLoads / 2);
        mma_rows<1, TM>(t, fa[1], fb[1]);
        __builtin_amdgcn_sched_barrier(0);
    }
    wait_vmem<0>();  // drain the over-issued loads before the stages are reused or released
}

template <typename CT> __device__ __forceinline__ void store_c(CT *p, float v);
// C is written once and not re-read by the kernel: stream it past the caches.
template <> __device__ __forceinline__ void store_c<float>(float *p, float v) { __builtin_nontemporal_store(v, p); }
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
