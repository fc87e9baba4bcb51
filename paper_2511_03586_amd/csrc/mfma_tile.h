// Shared bf16 MFMA main loops for gfx950: a workgroup of WM x WN wavefronts, each owning a
// (32*TM) x (32*TN) patch, computes a (32*TM*WM) x (32*TN*WN) tile of
//   sum_k A[m][k] * B[n][k]     with both operands K-contiguous
// ("matmul", "bmm" and "conv" rows of the operator table, Section 4.3 of the paper; the
// tiling / special-instruction / layout moves of Section 2.2 and the independent
// accumulator chains of Section 4.1 are applied by hand here).
//
// Two loops share the machinery (direct global->LDS loads into an XOR-swizzled ring, partial
// vmcnt waits, bare barriers, MFMAs interleaved one by one with the memory instructions):
//   * mfma_mainloop: K-step 32 (64-byte LDS rows, ring of NS stages (4, or as many as fit the
//     LDS for small tiles whose short steps cannot hide the memory latency), one barrier per step),
//     v_mfma_f32_32x32x16_bf16.  Any K that is a multiple of 32; the sources are objects, so
//     the implicit-GEMM convolution plugs its gathered operand in here.
//   * mfma_mainloop_k64: K-step 64 (128-byte LDS rows = whole cache lines per request, two
//     stages, one barrier per 64 K), v_mfma_f32_16x16x32_bf16.  Dense operands, K a multiple
//     of 64.  Measured ~5 % faster on 4096^3 (half the L2 requests and barriers).
#pragma once
#include <type_traits>
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
template <int TM, int TN, int WM, int WN, int NS = kStages>
struct TileShape {
    static constexpr int kWaves = WM * WN;
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    static constexpr int kLoadsA = BM / (16 * kWaves), kLoadsB = BN / (16 * kWaves);  // per lane per K-step
    static constexpr int kStageBytes = (BM + BN) * kRowBytes;
    static constexpr int kLdsBytes = NS * kStageBytes;  // NS = depth of the K-step-32 loop's ring
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
//   to NS-1 steps past the last one: a source must then keep naming readable (or out-of-range)
//   bytes; that data lands in a free stage and is never used, which keeps the number of
//   loads in flight, and so the vmcnt waits, uniform.
//   a_row0 / b_row0: first tile row of this wave's operands.  `wave` must be uniform.
//
// Schedule of step kt (operand registers F[kt&1] were filled during step kt-1):
//   wait until this wave's loads of step kt+1 have landed and its reads of stage kt are back;
//   barrier (now stage kt+1 is complete and stage kt is free for every wave);
//   read stage kt+1 into F[(kt+1)&1], refill stage kt with step kt+NS, and run the MFMAs of
//   step kt, the three instruction kinds interleaved.
template <int TM, int TN, int WM, int WN, int NS = kStages, typename SrcA, typename SrcB>
__device__ __forceinline__ void mfma_mainloop(WaveTile<TM, TN> &t, char *smem, int ktiles, int wave, int lane,
                                              int a_row0, int b_row0, SrcA &src_a, SrcB &src_b)
{
    using Shape = TileShape<TM, TN, WM, WN, NS>;
    constexpr int BM = Shape::BM;
    constexpr int kStageBytes = Shape::kStageBytes;
    constexpr int LA = Shape::kLoadsA, kLoads = Shape::kLoadsA + Shape::kLoadsB;
    static_assert(NS >= 3 && (NS & (NS - 1)) == 0, "ring depth: a power of two");
    static_assert((NS - 1) * kLoads < 64, "the loads in flight must fit the vmcnt counter");
    bf16x8_t fa[2][2][TM], fb[2][2][TN];  // [buffer][k-substep][tile]

    // loads of the sources' current K-step into ring slot kt % kStages; called with kt = 0, 1, 2, ...
    auto issue = [&](int kt) {
        char *stage = smem + (kt % NS) * kStageBytes;
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
        const char *stage = smem + (kt % NS) * kStageBytes;
        read_frags<TM, TN>(fa[buf][0], fb[buf][0], stage, stage + BM * kRowBytes, a_row0, b_row0, 0, lane);
        read_frags<TM, TN>(fa[buf][1], fb[buf][1], stage, stage + BM * kRowBytes, a_row0, b_row0, 1, lane);
    };
    auto step = [&](int kt, int buf) {
        wait_vmem_and_lds<(NS - 2) * kLoads>();
        wg_barrier();
        read_step(kt + 1, buf ^ 1);
        issue(kt + NS);
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

#pragma unroll
    for (int i = 0; i < NS; ++i) issue(i);
    wait_vmem<(NS - 1) * kLoads>();  // step 0 has landed
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

// ---- K-step 64, 16x16x32 MFMA ------------------------------------------------------
constexpr int kRowBytes64 = 128;  // 64 bf16 of K per LDS row: one cache line
// 16-byte chunk c (0..7) of tile row r is stored at chunk position c ^ swz64(r): 16 consecutive
// rows at one logical chunk land on the 16 distinct 16-byte slots of a 256-byte bank line.
__device__ __forceinline__ int swz64(int r) { return (r >> 1) & 7; }
__device__ __forceinline__ int frag_offset64(int row, int chunk) { return row * kRowBytes64 + ((chunk ^ swz64(row)) << 4); }

// One direct-to-LDS load of a wave (1 KiB = 8 rows of a stage) to `dst`.
__device__ __forceinline__ void issue_load_to(rsrc_t rsrc, uint32_t voffset, uint32_t soffset, char *dst)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void *)dst, 16, voffset, soffset, 0,
                                             0);
}

// Dense operand with K-contiguous rows, fetched 64 K at a time: load i of wave w fills tile
// rows (i*NW + w)*8 .. +7; lane l fetches row l/8, the chunk stored at position l%8.  Rows
// past `rows_valid` re-read the last valid row (their products are never stored).
template <int NLOADS, int NW>
struct RowMajorSrc64 {
    rsrc_t rsrc;
    uint32_t voff[NLOADS];
    uint32_t soff, soff_last;

    __device__ __forceinline__ RowMajorSrc64(const uint16_t *tile_base, int rows_valid, int64_t ld, int ksteps, int wave,
                                             int lane)
        : rsrc(make_rsrc(tile_base, (uint32_t)(((int64_t)(rows_valid - 1) * ld + (int64_t)ksteps * 64) * 2))), soff(0),
          soff_last((uint32_t)(ksteps - 1) * kRowBytes64)
    {
#pragma unroll
        for (int i = 0; i < NLOADS; ++i) {
            const int row = (i * NW + wave) * 8 + (lane >> 3);
            voff[i] = (uint32_t)(min(row, rows_valid - 1) * ld * 2) + (((lane & 7) ^ swz64(row)) << 4);
        }
    }
    // next K-step; past the last one it stays there
    __device__ __forceinline__ void advance() { soff = min(soff + (uint32_t)kRowBytes64, soff_last); }
};

template <int T16M, int T16N>  // 16x16 tiles per wave
struct WaveTile16 {
    float4_t acc[T16M][T16N];

    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int i = 0; i < T16M; ++i)
#pragma unroll
            for (int j = 0; j < T16N; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
    }
    // Must be called between the last mfma16() on this tile and the first ordinary (VALU, store)
    // read of `acc`: mfma16 is inline assembly, so the compiler's hazard recogniser does not see
    // the matrix instruction and inserts no wait states of its own; this supplies the 16+ the
    // hardware needs between an MFMA's issue and a VALU read of its result.
    __device__ __forceinline__ void finish() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }
};

// acc += a (16 n-rows x 32 k) * b (16 m-rows x 32 k)^T, in place.  Written as inline assembly
// because the compiler does not tie the destination of this 4-register MFMA to its
// accumulator input and then shuffles accumulators between the two register files (several
// hundred copies per K-step at this register pressure); "+a" pins each accumulator to its
// AGPRs.  The instruction is invisible to the hazard recogniser: every user calls
// WaveTile16::finish() behind its last mfma16 and before anything else reads the accumulators
// (mfma_mainloop_k64 does so on return; the 32x32x16 variant of the loop uses the builtin and is
// the cross-check in the tests).
__device__ __forceinline__ void mfma16(float4_t &acc, const bf16x8_t &a, const bf16x8_t &b)
{
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// K loop over `ksteps` steps of 64.  LDS: two stages of (BM + BN) rows x 128 bytes.
// Schedule of step p (stage p%2 holds it), in two halves of 32 K:
//   half 0: MFMAs on K 0..31 (fragments read during the previous half); in its first quarter
//           the fragments of K 32..63 are read from the same stage; at 3/8 a barrier (every
//           wave is done reading stage p), after which step p+2 starts loading into stage p;
//   between the halves: own loads of step p+1 have landed; barrier;
//   half 1: MFMAs on K 32..63; in its first quarter the first fragments of step p+1 are read
//           from the other stage; the rest of step p+2's loads.
// The loads of a step are thus spread over 5/8 of a half and a whole half instead of being
// issued by all four waves in one half: the texture path takes 64 bytes per clock, and a
// wave whose load cannot issue cannot issue the MFMAs behind it either (measured: 11 % fewer
// cycles on 4096^3).  The order is fixed by hand (scheduling fences), since the MFMAs are
// opaque to the scheduler.  The operands are
// swapped (B rows as the MFMA's row operand), so a lane ends up with 4 consecutive n of one m.
template <int TM, int TN, int WM, int WN, typename SrcA, typename SrcB>
__device__ __forceinline__ void mfma_mainloop_k64(WaveTile16<2 * TM, 2 * TN> &t, char *smem, int ksteps, int wave,
                                                  int lane, int a_row0, int b_row0, SrcA &src_a, SrcB &src_b)
{
    using Shape = TileShape<TM, TN, WM, WN>;
    constexpr int BM = Shape::BM, BN = Shape::BN, NW = Shape::kWaves;
    constexpr int kStageBytes64 = (BM + BN) * kRowBytes64;
    constexpr int LA = BM / (8 * NW), LB = BN / (8 * NW), kLoads = LA + LB;
    constexpr int T16M = 2 * TM, T16N = 2 * TN;
    constexpr int kMfmas = T16M * T16N;
    static_assert(2 * kStageBytes64 <= Shape::kLdsBytes, "the two stages fit the LDS the launch provides");
    static_assert(2 * kLoads < 64, "two steps of loads must fit the vmcnt counter");
    bf16x8_t fa[2][T16M], fb[2][T16N];  // [buffer][tile]: operands of one half-step

    // per-lane LDS byte offsets of the fragments of K half `half` (tile rows of 16, chunk = 4*half + lane/16)
    auto frag_a = [&](int i, int half) { return frag_offset64(a_row0 + i * 16 + (lane & 15), 4 * half + (lane >> 4)); };
    auto frag_b = [&](int j, int half) {
        return BM * kRowBytes64 + frag_offset64(b_row0 + j * 16 + (lane & 15), 4 * half + (lane >> 4));
    };
    auto issue_one = [&](char *stage, int i) {
        if (i < LA) {
            const uint32_t vo = src_a.voff[i], so = src_a.soff;
            issue_load_to(src_a.rsrc, vo, so, stage + (i * NW + wave) * 8 * kRowBytes64);
        } else {
            const uint32_t vo = src_b.voff[i - LA], so = src_b.soff;
            issue_load_to(src_b.rsrc, vo, so, stage + BM * kRowBytes64 + ((i - LA) * NW + wave) * 8 * kRowBytes64);
        }
    };
    // MFMAs of one half-step from fragment buffer BUF; between them: the reads of the next
    // half-step's fragments (stage rstage, K half RHALF) into the other buffer, the first
    // (half 0) or second (half 1) part of one step of global->LDS loads into lstage, and in
    // half 0 the barrier in front of those loads.
    // positions, in MFMAs of a half-step: reads before MFMA floor(g * kQ4 / kR), barrier of half
    // 0 before MFMA kQB, its kLa loads spread over [kQB, kMfmas), half 1's kLb loads over the half
    constexpr int kR = T16M + T16N, kQ4 = kMfmas / 4 > 0 ? kMfmas / 4 : 1, kQB = (3 * kMfmas) / 8;
    constexpr int kLa = kLoads / 2, kLb = kLoads - kLa, kSpan = kMfmas - kQB;
    auto half_step = [&](auto buf_c, auto rhalf_c, auto second_c, const char *rstage, char *lstage) {
        constexpr int BUF = decltype(buf_c)::value, RHALF = decltype(rhalf_c)::value;
        constexpr bool SECOND = decltype(second_c)::value;
#pragma unroll
        for (int q = 0; q < kMfmas; ++q) {
#pragma unroll
            for (int g = (q < kQ4 ? (q * kR + kQ4 - 1) / kQ4 : kR); g < (q < kQ4 ? ((q + 1) * kR + kQ4 - 1) / kQ4 : kR); ++g) {
                if (g < T16M)
                    fa[BUF ^ 1][g] = *reinterpret_cast<const bf16x8_t *>(rstage + frag_a(g, RHALF));
                else
                    fb[BUF ^ 1][g - T16M] = *reinterpret_cast<const bf16x8_t *>(rstage + frag_b(g - T16M, RHALF));
                __builtin_amdgcn_sched_barrier(0);
            }
            if (!SECOND && q == kQB) {
                wait_vmem_and_lds<kLoads>();  // own reads of this stage are back (the loads of step p+1 may still fly)
                wg_barrier();
            }
            if (!SECOND) {
#pragma unroll
                for (int i = (q >= kQB ? ((q - kQB) * kLa + kSpan - 1) / kSpan : kLa);
                     i < (q >= kQB ? ((q - kQB + 1) * kLa + kSpan - 1) / kSpan : kLa); ++i) {
                    issue_one(lstage, i);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int i = (q * kLb + kMfmas - 1) / kMfmas; i < ((q + 1) * kLb + kMfmas - 1) / kMfmas; ++i) {
                    issue_one(lstage, kLa + i);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            mfma16(t.acc[q / T16N][q % T16N], fb[BUF][q % T16N], fa[BUF][q / T16N]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using c0 = std::integral_constant<int, 0>;
    using c1 = std::integral_constant<int, 1>;

    for (int p = 0; p < 2; ++p) {  // steps 0 and 1 (step 1 may repeat step 0's data; it is then never used)
        char *stage = smem + p * kStageBytes64;
#pragma unroll
        for (int i = 0; i < kLoads; ++i) issue_one(stage, i);
        src_a.advance();
        src_b.advance();
    }
    wait_vmem<kLoads>();  // step 0 has landed
    wg_barrier();
#pragma unroll
    for (int i = 0; i < T16M; ++i) fa[0][i] = *reinterpret_cast<const bf16x8_t *>(smem + frag_a(i, 0));
#pragma unroll
    for (int j = 0; j < T16N; ++j) fb[0][j] = *reinterpret_cast<const bf16x8_t *>(smem + frag_b(j, 0));

    // (Steps are taken in pairs, so that the stage addresses are constants and a step boundary carries
    // no loop control: a 16-cycle MFMA hides three or four other instructions, not twenty.)
    auto k_step = [&](auto stage_c) {
        constexpr int ST = decltype(stage_c)::value;
        char *cur = smem + ST * kStageBytes64, *nxt = smem + (ST ^ 1) * kStageBytes64;
        wait_vmem_and_lds<kLoads>();  // the fragments of half 0 are back (loads of step p+1 may still fly)
        half_step(c0{}, c1{}, std::false_type{}, cur, cur);
        wait_vmem_and_lds<kLa>();  // own loads of step p+1 have landed (only this half's loads of step p+2 are younger)
        wg_barrier();
        half_step(c1{}, c0{}, std::true_type{}, nxt, cur);
        src_a.advance();
        src_b.advance();
    };
    int p = 0;
    for (; p + 1 < ksteps; p += 2) {
        k_step(c0{});
        k_step(c1{});
    }
    if (p < ksteps) k_step(c0{});
    wait_vmem_and_lds<0>();  // drain the over-issued loads and reads before LDS is reused or released
    t.finish();  // MFMA -> VALU read distance (see mfma16)
}

// The same loop and schedule with v_mfma_f32_32x32x16_bf16: 32 MFMAs of 32 cycles per half-step
// instead of 64 of 16, on 32x32 accumulators (the compiler ties those in place, so the plain
// builtin is used; A is the row operand, results are written by store_tile).  Per MAC the
// larger instruction reads half as many operand registers, and with random operands a
// register-only loop of it sustains 1.84 PFLOP/s on the box against 1.47 for 16x16x32: the
// clock is set by power, and this form needs less of it.
template <int TM, int TN, int WM, int WN, typename SrcA, typename SrcB>
__device__ __forceinline__ void mfma_mainloop_k64_mi32(WaveTile<TM, TN> &t, char *smem, int ksteps, int wave,
                                                       int lane, int a_row0, int b_row0, SrcA &src_a, SrcB &src_b)
{
    using Shape = TileShape<TM, TN, WM, WN>;
    constexpr int BM = Shape::BM, BN = Shape::BN, NW = Shape::kWaves;
    constexpr int kStageBytes64 = (BM + BN) * kRowBytes64;
    constexpr int LA = BM / (8 * NW), LB = BN / (8 * NW), kLoads = LA + LB;
    constexpr int kMfmas = 2 * TM * TN;  // per half-step: two k-substeps of 16 for every 32x32 accumulator
    static_assert(2 * kStageBytes64 <= Shape::kLdsBytes, "the two stages fit the LDS the launch provides");
    static_assert(2 * kLoads < 64, "two steps of loads must fit the vmcnt counter");
    bf16x8_t fa[2][2 * TM], fb[2][2 * TN];  // [buffer][k-substep * tiles + tile]: operands of one half-step

    // per-lane LDS byte offsets of fragment g of K half `half`: k-substep g / tiles of the half
    // (16 K: chunks 4*half + 2*(g / tiles) + lane/32), tile g % tiles (rows of 32)
    auto frag_a = [&](int g, int half) {
        return frag_offset64(a_row0 + (g % TM) * 32 + (lane & 31), 4 * half + 2 * (g / TM) + (lane >> 5));
    };
    auto frag_b = [&](int g, int half) {
        return BM * kRowBytes64 + frag_offset64(b_row0 + (g % TN) * 32 + (lane & 31), 4 * half + 2 * (g / TN) + (lane >> 5));
    };
    auto issue_one = [&](char *stage, int i) {
        if (i < LA) {
            const uint32_t vo = src_a.voff[i], so = src_a.soff;
            issue_load_to(src_a.rsrc, vo, so, stage + (i * NW + wave) * 8 * kRowBytes64);
        } else {
            const uint32_t vo = src_b.voff[i - LA], so = src_b.soff;
            issue_load_to(src_b.rsrc, vo, so, stage + BM * kRowBytes64 + ((i - LA) * NW + wave) * 8 * kRowBytes64);
        }
    };
    // MFMAs of one half-step from fragment buffer BUF; between them: the reads of the next
    // half-step's fragments (stage rstage, K half RHALF) into the other buffer, the first
    // (half 0) or second (half 1) part of one step of global->LDS loads into lstage, and in
    // half 0 the barrier in front of those loads.
    // positions, in MFMAs of a half-step: reads before MFMA floor(g * kQ4 / kR), barrier of half
    // 0 before MFMA kQB, its kLa loads spread over [kQB, kMfmas), half 1's kLb loads over the half
    constexpr int kFa = 2 * TM, kFb = 2 * TN;
    constexpr int kR = kFa + kFb, kQ4 = kMfmas / 4 > 0 ? kMfmas / 4 : 1, kQB = (3 * kMfmas) / 8;
    constexpr int kLa = kLoads / 2, kLb = kLoads - kLa, kSpan = kMfmas - kQB;
    auto half_step = [&](auto buf_c, auto rhalf_c, auto second_c, const char *rstage, char *lstage) {
        constexpr int BUF = decltype(buf_c)::value, RHALF = decltype(rhalf_c)::value;
        constexpr bool SECOND = decltype(second_c)::value;
#pragma unroll
        for (int q = 0; q < kMfmas; ++q) {
#pragma unroll
            for (int g = (q < kQ4 ? (q * kR + kQ4 - 1) / kQ4 : kR); g < (q < kQ4 ? ((q + 1) * kR + kQ4 - 1) / kQ4 : kR); ++g) {
                if (g < kFa)
                    fa[BUF ^ 1][g] = *reinterpret_cast<const bf16x8_t *>(rstage + frag_a(g, RHALF));
                else
                    fb[BUF ^ 1][g - kFa] = *reinterpret_cast<const bf16x8_t *>(rstage + frag_b(g - kFa, RHALF));
                __builtin_amdgcn_sched_barrier(0);
            }
            if (!SECOND && q == kQB) {
                wait_vmem_and_lds<kLoads>();  // own reads of this stage are back (the loads of step p+1 may still fly)
                wg_barrier();
            }
            if (!SECOND) {
#pragma unroll
                for (int i = (q >= kQB ? ((q - kQB) * kLa + kSpan - 1) / kSpan : kLa);
                     i < (q >= kQB ? ((q - kQB + 1) * kLa + kSpan - 1) / kSpan : kLa); ++i) {
                    issue_one(lstage, i);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int i = (q * kLb + kMfmas - 1) / kMfmas; i < ((q + 1) * kLb + kMfmas - 1) / kMfmas; ++i) {
                    issue_one(lstage, kLa + i);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            {
                // accumulator (i, j) takes its two k-substeps back to back
                const int ij = q / 2, ks = q % 2, i = ij / TN, j = ij % TN;
                t.acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[BUF][ks * TM + i], fb[BUF][ks * TN + j], t.acc[i][j], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using c0 = std::integral_constant<int, 0>;
    using c1 = std::integral_constant<int, 1>;

    for (int p = 0; p < 2; ++p) {  // steps 0 and 1 (step 1 may repeat step 0's data; it is then never used)
        char *stage = smem + p * kStageBytes64;
#pragma unroll
        for (int i = 0; i < kLoads; ++i) issue_one(stage, i);
        src_a.advance();
        src_b.advance();
    }
    wait_vmem<kLoads>();  // step 0 has landed
    wg_barrier();
#pragma unroll
    for (int i = 0; i < kFa; ++i) fa[0][i] = *reinterpret_cast<const bf16x8_t *>(smem + frag_a(i, 0));
#pragma unroll
    for (int j = 0; j < kFb; ++j) fb[0][j] = *reinterpret_cast<const bf16x8_t *>(smem + frag_b(j, 0));

    auto k_step = [&](auto stage_c) {  // (in pairs, as in mfma_mainloop_k64)
        constexpr int ST = decltype(stage_c)::value;
        char *cur = smem + ST * kStageBytes64, *nxt = smem + (ST ^ 1) * kStageBytes64;
        wait_vmem_and_lds<kLoads>();  // the fragments of half 0 are back (loads of step p+1 may still fly)
        half_step(c0{}, c1{}, std::false_type{}, cur, cur);
        wait_vmem_and_lds<kLa>();  // own loads of step p+1 have landed (only this half's loads of step p+2 are younger)
        wg_barrier();
        half_step(c1{}, c0{}, std::true_type{}, nxt, cur);
        src_a.advance();
        src_b.advance();
    };
    int p = 0;
    for (; p + 1 < ksteps; p += 2) {
        k_step(c0{});
        k_step(c1{});
    }
    if (p < ksteps) k_step(c0{});
    wait_vmem_and_lds<0>();  // drain the over-issued loads and reads before LDS is reused or released
}

// Write a wave's 16x16 accumulators to row-major C: element e of acc[i][j] is
// m = row0 + 16 i + lane%16, n = col0 + 16 j + 4 (lane/16) + e.  In the full-tile case pairs
// of column tiles are exchanged between the lanes of rows 0-7 and 8-15 of a 16-lane group
// (DPP row rotate by 8), so that one store instruction writes 8 rows of 32 contiguous
// elements (128 bytes of fp32) instead of 16 rows of 16.
// (A tile that was accumulated with mfma16 must have seen WaveTile16::finish() before this.)
template <int T16M, int T16N, typename CT>
__device__ __forceinline__ void store_tile16(const WaveTile16<T16M, T16N> &t, CT *C, int64_t ldc, int M, int N, int row0,
                                             int col0, float alpha, int lane)
{
    const int m16 = lane & 15, q = lane >> 4;
    const bool vec = ldc % 4 == 0 && (reinterpret_cast<uintptr_t>(C) & 15) == 0;
    if (vec && T16N % 2 == 0 && row0 + 16 * T16M <= M && col0 + 16 * T16N <= N) {
        const bool lo = m16 < 8;
#pragma unroll
        for (int i = 0; i < T16M; ++i) {
            CT *p = C + (int64_t)(row0 + 16 * i + (m16 & 7)) * ldc + col0 + (lo ? 0 : 16) + 4 * q;
#pragma unroll
            for (int j = 0; j < T16N; j += 2) {
                float4_t own0 = t.acc[i][j], own1 = t.acc[i][j + 1];
                own0 *= alpha;
                own1 *= alpha;
                float4_t s1, s2;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x = lo ? own1[e] : own0[e];
                    const float y = dpp_move<0x128>(x);  // row_ror:8 -> the value of lane ^ 8
                    s1[e] = lo ? own0[e] : y;
                    s2[e] = lo ? y : own1[e];
                }
                if constexpr (sizeof(CT) == 4) {
                    __builtin_nontemporal_store(s1, reinterpret_cast<float4_t *>(p + 16 * j));
                    __builtin_nontemporal_store(s2, reinterpret_cast<float4_t *>(p + 16 * j + 8 * ldc));
                } else {
                    *reinterpret_cast<uint2_t *>(p + 16 * j) = uint2_t{pack_bf16(s1[0], s1[1]), pack_bf16(s1[2], s1[3])};
                    *reinterpret_cast<uint2_t *>(p + 16 * j + 8 * ldc) =
                        uint2_t{pack_bf16(s2[0], s2[1]), pack_bf16(s2[2], s2[3])};
                }
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < T16M; ++i)
#pragma unroll
            for (int j = 0; j < T16N; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int m = row0 + 16 * i + m16, n = col0 + 16 * j + 4 * q + e;
                    if (m < M && n < N) store_c<CT>(C + (int64_t)m * ldc + n, alpha * t.acc[i][j][e]);
                }
    }
}

// bf16 variant of the full-tile write-out: the wave's tile is packed to bf16 and staged in a
// private LDS region (rows of 32*T16N bytes, 16-byte chunks XOR-swizzled by the row so that
// neither the column-wise writes nor the row-wise reads conflict), then written as 16 bytes
// per lane, whole rows of the tile per group of 2*T16N lanes.  `stage` must not be in use by
// any other wave (the caller puts a barrier between the main loop and this).
// Returns false (nothing written) when the tile is not full or C is not 16-byte aligned.
template <int T16M, int T16N>
__device__ __forceinline__ bool store_tile16_bf16(const WaveTile16<T16M, T16N> &t, uint16_t *C, int64_t ldc, int M, int N,
                                                  int row0, int col0, float alpha, int lane, char *stage)
{
    constexpr int kRowBytes = 32 * T16N, kChunks = 2 * T16N, kMask = (kChunks < 16 ? kChunks : 16) - 1;
    static_assert((kChunks & (kChunks - 1)) == 0 && 64 % kChunks == 0, "power-of-two chunks per row");
    if (!(ldc % 8 == 0 && (reinterpret_cast<uintptr_t>(C) & 15) == 0 && row0 + 16 * T16M <= M && col0 + 16 * T16N <= N))
        return false;
    const int m16 = lane & 15, q = lane >> 4;
#pragma unroll
    for (int i = 0; i < T16M; ++i) {
        const int row = 16 * i + m16;
#pragma unroll
        for (int j = 0; j < T16N; ++j) {
            const float4_t v = t.acc[i][j] * alpha;
            const int chunk = (2 * j + (q >> 1)) ^ (row & kMask);  // 8 bf16 per chunk: columns 16 j + 8 (q/2) ..
            *reinterpret_cast<uint2_t *>(stage + row * kRowBytes + chunk * 16 + (q & 1) * 8) =
                uint2_t{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        }
    }
    // (same wave wrote and reads: the LDS operations of a wave complete in order)
    constexpr int kRowsPerInstr = 64 / kChunks;
#pragma unroll
    for (int r0 = 0; r0 < 16 * T16M; r0 += kRowsPerInstr) {
        const int row = r0 + lane / kChunks, c = lane % kChunks;
        const uint4_t v = *reinterpret_cast<const uint4_t *>(stage + row * kRowBytes + ((c ^ (row & kMask)) * 16));
        __builtin_nontemporal_store(v, reinterpret_cast<uint4_t *>(C + (int64_t)(row0 + row) * ldc + col0 + c * 8));
    }
    return true;
}

}  // namespace perf
