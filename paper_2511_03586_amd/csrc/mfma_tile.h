// Shared bf16 MFMA main loop for gfx950: a workgroup of WM x WN wavefronts, each owning
// TM x TN MFMA tiles of 32x32, computes a (32*TM*WM) x (32*TN*WN) tile of
// sum_k A[m][k] * B[n][k]  with both operands K-contiguous
// ("matmul", "bmm" and "conv" rows of the operator table, Section 4.3 of the paper; the
// tiling / special-instruction / layout moves of Section 2.2 and the independent
// accumulator chains of Section 4.1 are applied by hand here).
//
// Data path per K-step of 32:
//   L2 --buffer_load_dwordx4 ... lds--> LDS ring of 4 stages (XOR-swizzled 16-byte chunks)
//   LDS --ds_read_b128--> operand registers (double buffered per K-step)
//   v_mfma_f32_32x32x16_bf16 into TM*TN independent 32x32 fp32 accumulators per wave.
// Loads run several K-steps ahead of the MFMAs and are issued between them, so the
// L2 -> LDS stream is continuous; the wait before a step's barrier is a partial vmcnt that
// leaves the younger steps in flight.  One workgroup barrier per K-step.
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
    uint32_t soff, soff_last;

    __device__ __forceinline__ RowMajorSrc(const uint16_t *tile_base, int rows_valid, int64_t ld, int ktiles, int wave,
                                           int lane)
        : rsrc(make_rsrc(tile_base, (uint32_t)(((int64_t)(rows_valid - 1) * ld + (int64_t)ktiles * kBK) * 2))),
          soff(0), soff_last((uint32_t)(ktiles - 1) * kRowBytes)
    {
#pragma unroll
        for (int i = 0; i < NLOADS; ++i) {
            const int row = load_row<NW>(i, wave, lane);
            voff[i] = (uint32_t)(min(row, rows_valid - 1) * ld * 2) + load_chunk(row, lane) * 16;
        }
    }
    __device__ __forceinline__ uint32_t voffset(int i) const { return voff[i]; }
    __device__ __forceinline__ uint32_t soffset() const { return soff; }
    // next K-step; past the last one it stays there
    __device__ __forceinline__ void advance() { soff = min(soff + (uint32_t)kRowBytes, soff_last); }
};

// All MFMAs of one K-step (two 16-wide k-substeps).  The two substeps of an accumulator
// are issued back to back: consecutive MFMAs on the same accumulator forward it inside the
// matrix pipe instead of going through the register file, which measurably lowers power
// (the chip is power-limited under MFMA load, so lower energy per MFMA is a higher clock).
template <int TM, int TN>
__device__ __forceinline__ void mma_kstep(WaveTile<TM, TN> &t, const bf16x8_t (&a)[2][TM], const bf16x8_t (&b)[2][TN])
{
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            t.acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[0][j], t.acc[i][j], 0, 0, 0);
            t.acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][i], b[1][j], t.acc[i][j], 0, 0, 0);
        }
}

// K loop shared by GEMM and implicit-GEMM convolution.
//   SrcA / SrcB describe where an operand's stage comes from and walk the K-steps in
//   order: a buffer resource `rsrc`, voffset(i) = per-lane byte offset of the 16-byte chunk
//   fetched by load i (0 .. kLoadsA-1 / kLoadsB-1) of the current step, soffset() = uniform
//   byte offset of the current step, advance() = go to the next step.  The loop advances up
//   to 3 steps past the last one: a source must then keep naming readable (or out-of-range)
//   bytes; that data lands in a free stage and is never used, which keeps the number of
//   loads in flight, and so the vmcnt waits, uniform.
//   a_row0 / b_row0: first tile row of this wave's operands.  `wave` must be uniform.
//
// Schedule of step kt (operand registers F[kt&1] were filled during step kt-1):
//   wait until this wave's loads of step kt+1 have landed and its reads of stage kt are back;
//   barrier (now stage kt+1 is complete and stage kt is free for every wave);
//   read stage kt+1 into F[(kt+1)&1], refill stage kt with step kt+4, and run the MFMAs of
//   step kt, the three instruction kinds interleaved.
template <int TM, int TN, int WM, int WN, typename SrcA, typename SrcB>
__device__ __forceinline__ void mfma_mainloop(WaveTile<TM, TN> &t, char *smem, int ktiles, int wave, int lane,
                                              int a_row0, int b_row0, SrcA &src_a, SrcB &src_b)
{
    using Shape = TileShape<TM, TN, WM, WN>;
    constexpr int BM = Shape::BM;
    constexpr int kStageBytes = Shape::kStageBytes;
    constexpr int LA = Shape::kLoadsA, kLoads = Shape::kLoadsA + Shape::kLoadsB;
    static_assert(3 * kLoads < 64, "three K-steps of loads must fit the vmcnt counter");
    bf16x8_t fa[2][2][TM], fb[2][2][TN];  // [buffer][k-substep][tile]

    // loads of the sources' current K-step into ring slot kt % kStages; called with kt = 0, 1, 2, ...
    auto issue = [&](int kt) {
        char *stage = smem + (kt % kStages) * kStageBytes;
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            if (i < LA)
                issue_load<Shape::kWaves>(src_a.rsrc, src_a.voffset(i), src_a.soffset(), stage, i, wave);
            else
                issue_load<Shape::kWaves>(src_b.rsrc, src_b.voffset(i - LA), src_b.soffset(), stage + BM * kRowBytes,
                                          i - LA, wave);
        }
        src_a.advance();
        src_b.advance();
    };
    auto read_step = [&](int kt, int buf) {
        const char *stage = smem + (kt % kStages) * kStageBytes;
        read_frags<TM, TN>(fa[buf][0], fb[buf][0], stage, stage + BM * kRowBytes, a_row0, b_row0, 0, lane);
        read_frags<TM, TN>(fa[buf][1], fb[buf][1], stage, stage + BM * kRowBytes, a_row0, b_row0, 1, lane);
    };
    auto step = [&](int kt, int buf) {
        wait_vmem_and_lds<2 * kLoads>();
        wg_barrier();
        read_step(kt + 1, buf ^ 1);
        issue(kt + 4);
        mma_kstep<TM, TN>(t, fa[buf], fb[buf]);
        // interleave: one LDS read or one buffer load behind each of the first MFMAs
#pragma unroll
        for (int g = 0; g < 2 * (TM + TN); ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
        }
#pragma unroll
        for (int g = 0; g < kLoads; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    issue(0);
    issue(1);
    issue(2);
    issue(3);
    wait_vmem<3 * kLoads>();  // step 0 has landed
    wg_barrier();
    read_step(0, 0);

    int kt = 0;
    for (; kt + 1 < ktiles; kt += 2) {
        step(kt, 0);
        step(kt + 1, 1);
    }
    if (kt < ktiles) step(kt, 0);
    wait_vmem_and_lds<0>();  // drain the over-issued loads and reads before LDS is reused or released
}

// Ping-pong K loop for workgroups of two wave groups (WM == 2; group = wave / WN, so the
// two waves that share a SIMD belong to different groups).  Each K-step of a wave is split
// into a memory phase (all operand reads of the step, the global->LDS loads of step kt+3,
// the waits) and a compute phase (only MFMAs, from registers).  The groups run half a
// period apart: while one group's MFMAs own the matrix pipe, the other group does its
// memory phase, so load issue, LDS latency and barrier waits hide behind MFMAs.  Barriers
// separate the phases; group 1 executes one extra barrier before the loop (which shifts
// its phase) and group 0 one after it, so every wave executes the same number.
//
// Stage safety (ring of 4, loads 3 steps ahead): the loads of step kt+3 overwrite the
// stage of step kt-1.  A wave issues them in its memory phase kt, which starts after a
// barrier that every wave reaches only when its own reads of stage kt-1 have returned
// (lgkmcnt(0) ends each memory phase).  A wave reads stage kt after a barrier that every
// wave reaches only when its own loads of step kt have landed (the vmcnt wait that ends
// memory phase kt-1 leaves just two younger steps in flight).
template <int TM, int TN, int WM, int WN, typename SrcA, typename SrcB>
__device__ __forceinline__ void mfma_mainloop_pingpong(WaveTile<TM, TN> &t, char *smem, int ktiles, int wave,
                                                       int lane, int a_row0, int b_row0, SrcA &src_a, SrcB &src_b)
{
    using Shape = TileShape<TM, TN, WM, WN>;
    static_assert(WM == 2, "two wave groups");
    constexpr int BM = Shape::BM;
    constexpr int kStageBytes = Shape::kStageBytes;
    constexpr int LA = Shape::kLoadsA, kLoads = Shape::kLoadsA + Shape::kLoadsB;
    static_assert(2 * kLoads < 64, "two K-steps of loads must fit the vmcnt counter");
    const int group = wave / WN;  // uniform
    bf16x8_t fa[2][TM], fb[2][TN];

    // loads of the sources' current K-step into ring slot kt % kStages; called with kt = 0, 1, 2, ...
    auto issue = [&](int kt) {
        char *stage = smem + (kt % kStages) * kStageBytes;
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            if (i < LA)
                issue_load<Shape::kWaves>(src_a.rsrc, src_a.voffset(i), src_a.soffset(), stage, i, wave);
            else
                issue_load<Shape::kWaves>(src_b.rsrc, src_b.voffset(i - LA), src_b.soffset(), stage + BM * kRowBytes,
                                          i - LA, wave);
        }
        src_a.advance();
        src_b.advance();
    };

    issue(0);
    issue(1);
    issue(2);
    wait_vmem<2 * kLoads>();  // own part of step 0 has landed
    wg_barrier();
    if (group == 1) wg_barrier();  // phase shift; balanced by group 0's barrier after the loop

    for (int kt = 0; kt < ktiles; ++kt) {
        const char *cur = smem + (kt % kStages) * kStageBytes;
        // memory phase
        read_frags<TM, TN>(fa[0], fb[0], cur, cur + BM * kRowBytes, a_row0, b_row0, 0, lane);
        read_frags<TM, TN>(fa[1], fb[1], cur, cur + BM * kRowBytes, a_row0, b_row0, 1, lane);
        issue(kt + 3);
        wait_vmem_and_lds<2 * kLoads>();  // own loads of step kt+1 landed, own reads returned
        __builtin_amdgcn_sched_barrier(0);
        wg_barrier();
        // compute phase
        __builtin_amdgcn_s_setprio(1);
        mma_kstep<TM, TN>(t, fa, fb);
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        wg_barrier();
    }
    if (group == 0) wg_barrier();
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
