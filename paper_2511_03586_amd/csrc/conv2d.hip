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
//  * conv2d_wreg_kernel: bf16, 3x3 filter, 64 -> 128 channels: weights held in registers.
//  * conv2d_wres_kernel: the same with the input rows of a workgroup's pixel range resident in
//    LDS (stride 1, ranges inside one image, rows that fit): the benchmark's shape.
//  * conv2d_mfma_kernel: bf16, C a multiple of 32; main loop shared with the GEMM.
//  * conv2d_rowmfma_kernel: few input channels with S*C <= 16 (e.g. the 3-channel 5x5 first
//    layer of the paper's "conv 1"): one filter row per 16-wide MFMA K-step, stride 1.
//  * conv2d_smallc_kernel: other few-channel cases: one thread per output pixel and block of
//    KB output channels, weights broadcast from LDS, fp32 FMAs.
//  * conv2d_direct_kernel: any other legal case; one thread per output element.
#include <atomic>
#include "mfma_tile.h"
#include "f32mfma.h"
#include "host_utils.h"
#include "timeline.h"
#include <algorithm>
#include <utility>

namespace perf {

struct ConvGeom {
    int N, H, W, C, K, R, S, sh, sw, ph, pw, P, Q;
};

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a
// compile-time constant inside the body (template arguments, register-array indices).
template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F &&f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F &&>(f));
}

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
        int H, W, C, R, S, cblocks;
        int r, s, cb;  // filter tap and channel block of the current K-step (uniform)
        __device__ __forceinline__ uint32_t voffset(int i) const
        {
            const int ih = ih0[i] + r, iw = iw0[i] + s;
            const bool inside = ih >= 0 && ih < H && iw >= 0 && iw < W;
            const int64_t off = pix_off[i] + ((int64_t)(r * W + s) * C + cb * kBK) * 2;
            return inside ? (uint32_t)off : kOutOfRange;
        }
        __device__ __forceinline__ uint32_t soffset() const { return 0; }
        // next K-step: channel block fastest, then s, then r; past the last step it stays there
        __device__ __forceinline__ void advance()
        {
            if (r == R - 1 && s == S - 1 && cb == cblocks - 1) return;
            if (++cb == cblocks) {
                cb = 0;
                if (++s == S) {
                    s = 0;
                    ++r;
                }
            }
        }
    };
    ActSrc src_a{make_rsrc(x, (uint32_t)((int64_t)g.N * g.H * g.W * g.C * 2)), {}, {}, {}, g.H, g.W, g.C, g.R, g.S,
                 cblocks, 0, 0, 0};
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
    RowMajorSrc<LB, NW> src_b(w + (int64_t)n0 * ldb, min(BN, g.K - n0), ldb, ktiles, wave, lane);

    WaveTile<TM, TN> t;
    t.clear();
    const int a_row0 = wm * 32 * TM, b_row0 = wn * 32 * TN;
    mfma_mainloop<TM, TN, WM, WN>(t, smem, ktiles, wave, lane, a_row0, b_row0, src_a, src_b);
    store_tile<TM, TN, CT>(t, y, g.K, Mtot, g.K, m0 + a_row0, n0 + b_row0, 1.0f, lane);
}

// ---- weights-in-registers kernel ---------------------------------------------------
// Stage one accumulator (32 channels x 32 pixels, weights as the MFMA row operand) for the
// row-wise write-out: element group a of a lane is 4 consecutive channels of its pixel.
template <typename CT>
__device__ __forceinline__ void stage_acc(const float16_t &acc, char *stg)
{
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        if constexpr (sizeof(CT) == 4) {
            *reinterpret_cast<float4_t *>(stg + 8 * a * 4) = float4_t{acc[4 * a], acc[4 * a + 1], acc[4 * a + 2], acc[4 * a + 3]};
        } else {
            *reinterpret_cast<uint2_t *>(stg + 8 * a * 2) =
                uint2_t{pack_bf16(acc[4 * a], acc[4 * a + 1]), pack_bf16(acc[4 * a + 2], acc[4 * a + 3])};
        }
    }
}

// Weights of one MFMA wave's 32 output channels -> registers (both weights-in-registers
// kernels).  Fragment kk covers K indices kk*16 .. +15 of the filter (r, s, c order); a lane
// holds channel lane%32 and the 8 K values starting at 8*(lane/32).  Read straight from
// memory that pattern touches 32 different rows per instruction, so the wave's 36 KiB go
// through a private LDS region (`region` + wave * 2 * kQBytes, 18 KiB per wave) with coalesced
// global->LDS loads, in four quarters of R*S*C/4 K values through two sub-regions, so that
// two quarters are always in flight while a third is read into registers.  A row's chunks of
// 16 bytes are stored rotated by row/8 chunks, which spreads the 16 rows read by one
// ds_read_b128 phase over all 16 bank slots (row pitch 18 chunks = 2 slots).
template <int R, int S, int C>
__device__ __forceinline__ void load_weight_frags(bf16x8_t (&wf)[R * S * C / 16], char *region, const uint16_t *w,
                                                  int wave, int lane)
{
    constexpr int KSUB = R * S * C / 16;
    constexpr int kQC = R * S * C / 32;       // 16-byte chunks per weight row and quarter (18)
    constexpr int kQLoads = 32 * kQC / 64;    // wave loads per quarter (9)
    constexpr int kQBytes = 32 * kQC * 16;
    static_assert((32 * kQC) % 64 == 0 && KSUB % 4 == 0 && R * S * C == 32 * kQC, "whole wave loads per quarter");
    char *wreg = region + wave * (2 * kQBytes);
    const rsrc_t wr = make_rsrc(w + (int64_t)wave * 32 * (R * S * C), (uint32_t)(32 * R * S * C * 2));
    uint32_t wvo[kQLoads];
#pragma unroll
    for (int i = 0; i < kQLoads; ++i) {
        const int L = i * 64 + lane, row = L / kQC;
        int c = L % kQC - (row >> 3);
        c = c < 0 ? c + kQC : c;
        wvo[i] = (uint32_t)(row * (4 * kQC) + c) * 16u;
    }
    const int frow = lane & 31;
    auto issue_q = [&](int q, int sub) {
#pragma unroll
        for (int i = 0; i < kQLoads; ++i) {
            const uint32_t vo = wvo[i];
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (__attribute__((address_space(3))) void *)(wreg + sub * kQBytes + i * 1024),
                                                     16, vo, q * (kQC * 16), 0, 0);
        }
    };
    auto read_q = [&](int q, int sub) {
#pragma unroll
        for (int kk = 0; kk < KSUB / 4; ++kk) {
            int p = 2 * kk + (lane >> 5) + (frow >> 3);
            p = p >= kQC ? p - kQC : p;
            wf[q * (KSUB / 4) + kk] = *reinterpret_cast<const bf16x8_t *>(wreg + sub * kQBytes + (frow * kQC + p) * 16);
        }
    };
    issue_q(0, 0);
    issue_q(1, 1);
    wait_vmem<kQLoads>();
    read_q(0, 0);
    wait_vmem_and_lds<kQLoads>();
    issue_q(2, 0);
    wait_vmem<kQLoads>();
    read_q(1, 1);
    wait_vmem_and_lds<kQLoads>();
    issue_q(3, 1);
    wait_vmem<kQLoads>();
    read_q(2, 0);
    wait_vmem<0>();
    read_q(3, 1);
    wait_vmem_and_lds<0>();
}

// For filters small enough that a wavefront can keep its share of them in registers
// (here: 128 output channels, 4 waves x 32 channels, R*S*C = 576 -> 36 operand fragments
// = 144 VGPRs per lane), the contraction is turned around: the weights never move after
// the prologue, and the activations stream through LDS once per 32-pixel block.
// One persistent workgroup of 8 waves per CU owns a contiguous range of output pixels; the
// waves are specialised, and a SIMD hosts one of each kind:
//   * waves 0-3 ("MFMA waves") hold the weights of 32 output channels each.  Per block
//     they read the whole 32 x 576 im2col slice from an LDS ring slot (one ds_read_b128
//     per MFMA, through a rolling window of 9 operand registers) and chain 36 MFMAs on one
//     accumulator; the previous block's results are converted and staged in LDS in the
//     shadow of the first MFMAs.  Nothing else is in their instruction stream.
//   * waves 4-7 ("memory waves") compute the im2col offsets, fetch each block's slice
//     global -> LDS three blocks ahead (zero padding by the buffer range check, as R*S*C/32
//     swizzled sub-tiles of 32 pixels x 32 channels), and write staged results out as
//     whole pixel rows, 16 bytes per lane.
//   * one workgroup barrier per block, three quarters into its MFMAs, when the operand
//     window moves on to the next block's slot.
// The MFMA takes the weights as its row operand, so a lane ends up with 4 consecutive
// output channels of one pixel.
template <int R, int S, int C, typename CT>
__global__ __launch_bounds__(512) void conv2d_wreg_kernel(const uint16_t *__restrict__ x,
                                                          const uint16_t *__restrict__ w, CT *__restrict__ y,
                                                          ConvGeom g, int px_per_wg)
{
    constexpr int KOUT = 128;               // 4 MFMA waves x 32 channels
    constexpr int KSUB = R * S * C / 16;    // MFMA k-substeps per pixel block
    constexpr int CB = C / 32;              // 32-channel sub-tiles per filter tap
    constexpr int NSUB = R * S * CB;        // LDS sub-tiles per block, 2 KiB each
    constexpr int kSlot = NSUB * 2048;
    constexpr int kSlots = 3;
    constexpr int kLoads = NSUB * 2 / 4;    // direct-to-LDS loads per memory wave per block (1 KiB each)
    // output staging: a block's 32 x 128 results go through LDS so that global stores write
    // whole pixel rows (16 bytes per lane); the row pitch is padded by 16 bytes against bank
    // conflicts of the column-wise writes
    constexpr int kOutPitch = KOUT * (int)sizeof(CT) + 16;
    constexpr int kOutBytes = 32 * kOutPitch;
    constexpr int kRowLanes = KOUT * (int)sizeof(CT) / 16;  // lanes per pixel row of 16-byte pieces
    constexpr int kStores = 8 * kRowLanes / 64;             // store instructions per memory wave per block (8 rows each)
    constexpr int kWin = 9;                                 // operand window of the MFMA waves
    static_assert(CB == 2, "two 32-channel sub-tiles per filter tap");
    static_assert((NSUB * 2) % 4 == 0, "sub-tiles must divide among the four memory waves");
    static_assert(KSUB % kWin == 0 && KSUB % 4 == 0, "window and weight quarters must divide the fragment count");
    static_assert(kLoads + 2 * kStores < 64, "vmcnt is a 6-bit counter");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    char *const out_stage = smem + kSlots * kSlot;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int Mtot = g.N * g.P * g.Q;
    // workgroup ids are dealt round-robin to the 8 XCDs: give each XCD a contiguous run of pixel
    // ranges, so that neighbouring ranges (which share halo rows of the input) share an L2
    const int wg = gridDim.x % 8 == 0 ? (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
    const int start = wg * px_per_wg, end = min(start + px_per_wg, Mtot);
    const int nblocks = (end - start + 31) / 32;
    // Both kinds of wave execute exactly 2 + nblocks workgroup barriers.

    if (wave < 4) {
        // ------------------------------ MFMA waves ------------------------------
        __builtin_amdgcn_s_setprio(2);
        // Weights of this wave's 32 channels -> registers, through a private LDS region that
        // overlaps ring slot 2 and the output staging, which are not in use before the first
        // barrier; slots 0 and 1 are being filled by the memory waves meanwhile.
        bf16x8_t wf[KSUB];
        load_weight_frags<R, S, C>(wf, smem + 2 * kSlot, w, wave, lane);
        const int frag_lo = frag_offset(lane & 31, lane >> 5);        // k-substep 0 of a sub-tile
        const int frag_hi = frag_offset(lane & 31, 2 + (lane >> 5));  // k-substep 1
        // fragment kk of a block: sub-tile kk/2 (32 channels = 2 k-substeps; sub-tiles are stored
        // tap-major), read relative to the two per-lane addresses of the block's slot so that
        // the sub-tile offset fits the instruction's immediate field
        typedef const __attribute__((address_space(3))) char lds_char_t;
        typedef const __attribute__((address_space(3))) bf16x8_t lds_frag_t;
        lds_char_t *const lds0 = (lds_char_t *)smem;
        auto read_frag = [&](uint32_t slot_lo, uint32_t slot_hi, int kk) {
            return *(lds_frag_t *)(lds0 + ((kk & 1) ? slot_hi : slot_lo) + (kk / 2) * 2048);
        };
        // staging position: lane holds channels wave*32 + 8a + 4*(lane/32) + 0..3 of pixel lane%32
        const int stage_wr = (lane & 31) * kOutPitch + (wave * 32 + 4 * (lane >> 5)) * (int)sizeof(CT);

        wg_barrier();  // block 0 is complete in slot 0 (and every wave is done with the weight region)
        bf16x8_t af[kWin];
#pragma unroll
        for (int kk = 0; kk < kWin; ++kk) af[kk] = read_frag((uint32_t)frag_lo, (uint32_t)frag_hi, kk);
        float16_t accs[2];
#pragma unroll
        for (int e = 0; e < 16; ++e) accs[0][e] = accs[1][e] = 0.f;

        // One block: `acc` collects block b, `prev` holds block b-1's results (zeros for b = 0,
        // staged but never written out).  In the shadow of the first MFMAs `prev` is converted
        // and staged, then cleared for block b+1.  Before the barrier every read of this
        // block's slot has returned; after it block b+1 is complete in LDS.
        // (blocks come in pairs that swap the two accumulators; the pair is the loop's unit, so that a block
        // boundary carries no loop control)
        auto do_block = [&](int b, auto hc) {
            constexpr int h = decltype(hc)::value;
            float16_t &acc = accs[h];
            float16_t &prev = accs[h ^ 1];
            const uint32_t cur = (uint32_t)(b % kSlots) * kSlot, nxt = (uint32_t)((b + 1) % kSlots) * kSlot;
            uint32_t cur_lo = cur + frag_lo, cur_hi = cur + frag_hi;
            uint32_t nxt_lo = nxt + frag_lo, nxt_hi = nxt + frag_hi;
            // opaque to the optimiser: folded with the sub-tile offsets they turn into one address
            // register per read, which does not fit the register budget of two waves per SIMD
            asm volatile("" : "+v"(cur_lo), "+v"(cur_hi), "+v"(nxt_lo), "+v"(nxt_hi));
            char *stg = out_stage + ((b - 1) & 1) * kOutBytes + stage_wr;
#pragma unroll
            for (int kk = 0; kk < KSUB - kWin; ++kk) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[kk], af[kk % kWin], acc, 0, 0, 0);
                af[kk % kWin] = read_frag(cur_lo, cur_hi, kk + kWin);
                if (kk >= 1 && kk < 5) {
                    const int a = kk - 1;
                    if constexpr (sizeof(CT) == 4) {
                        *reinterpret_cast<float4_t *>(stg + 8 * a * 4) =
                            float4_t{prev[4 * a], prev[4 * a + 1], prev[4 * a + 2], prev[4 * a + 3]};
                    } else {
                        *reinterpret_cast<uint2_t *>(stg + 8 * a * 2) =
                            uint2_t{pack_bf16(prev[4 * a], prev[4 * a + 1]), pack_bf16(prev[4 * a + 2], prev[4 * a + 3])};
                    }
                }
                if (kk >= 6 && kk < 10) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) prev[4 * (kk - 6) + e] = 0.f;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            wait_vmem_and_lds<0>();
            wg_barrier();
#pragma unroll
            for (int kk = KSUB - kWin; kk < KSUB; ++kk) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[kk], af[kk % kWin], acc, 0, 0, 0);
                af[kk % kWin] = read_frag(nxt_lo, nxt_hi, kk + kWin - KSUB);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        int b0 = 0;
        for (; b0 + 1 < nblocks; b0 += 2) {
            do_block(b0, std::integral_constant<int, 0>{});
            do_block(b0 + 1, std::integral_constant<int, 1>{});
        }
        if (b0 < nblocks) do_block(b0, std::integral_constant<int, 0>{});
        // the last block's results
        const float16_t last = ((nblocks - 1) & 1) ? accs[1] : accs[0];
        stage_acc<CT>(last, out_stage + ((nblocks - 1) & 1) * kOutBytes + stage_wr);
        wait_vmem_and_lds<0>();
        wg_barrier();
    } else {
        // ------------------------------ memory waves ------------------------------
        const int mw = wave - 4;
        // activation loads: a wave fills half `mw % 2` (16 pixels) of sub-tiles mw/2, mw/2 + 2, ...
        // lane -> pixel row half*16 + lane/4 of the block, chunk position lane%4
        const rsrc_t xr = make_rsrc(x, (uint32_t)((int64_t)g.N * g.H * g.W * g.C * 2));
        const int half = mw & 1, row_l = half * 16 + (lane >> 2);
        int n_l, p_l, q_l;  // pixel start + row_l of block 0 as (image, output row, output column)
        {
            const int m = start + row_l;
            n_l = m / (g.P * g.Q);
            const int pq = m - n_l * (g.P * g.Q);
            p_l = pq / g.Q;
            q_l = pq - p_l * g.Q;
        }
        int m_l = start + row_l;
        const uint32_t chunk_l = load_chunk(row_l, lane) * 16;
        // All offsets are 32-bit: the host admits this kernel only for tensors below 2 GiB, and
        // an offset is used only when its tap lies inside the image (then it is the true one).
        uint32_t voff_l[kLoads];  // per-lane offsets of the next block to fetch (out of range: zeros)
        auto prep_block = [&]() {
            const int ih0 = p_l * g.sh - g.ph, iw0 = q_l * g.sw - g.pw;
            const uint32_t pix = (uint32_t)(((n_l * g.H + ih0) * g.W + iw0) * C) * 2u + chunk_l;
            // row / column validity once per filter row / column
            bool row_ok[R], col_ok[S];
#pragma unroll
            for (int r = 0; r < R; ++r) row_ok[r] = m_l < end && (unsigned)(ih0 + r) < (unsigned)g.H;
#pragma unroll
            for (int sft = 0; sft < S; ++sft) col_ok[sft] = (unsigned)(iw0 + sft) < (unsigned)g.W;
#pragma unroll
            for (int t = 0; t < kLoads; ++t) {
                // sub-tile 2t + mw/2 = filter tap t, channel block mw/2
                const int r = t / S, sft = t % S;
                const uint32_t tap_off = (uint32_t)((r * g.W + sft) * C + (mw >> 1) * 32) * 2u;  // scalar
                voff_l[t] = (row_ok[r] && col_ok[sft]) ? pix + tap_off : kOutOfRange;
            }
            // advance this lane's pixel by one block (32 pixels): Q >= 32 (checked by the host),
            // so the column wraps at most once
            m_l += 32;
            q_l += 32;
            const bool wrap_q = q_l >= g.Q;
            q_l = wrap_q ? q_l - g.Q : q_l;
            p_l = wrap_q ? p_l + 1 : p_l;
            const bool wrap_p = p_l == g.P;
            p_l = wrap_p ? 0 : p_l;
            n_l = wrap_p ? n_l + 1 : n_l;
        };
        auto fire_block = [&](int b) {
            char *slot = smem + (b % kSlots) * kSlot;
#pragma unroll
            for (int t = 0; t < kLoads; ++t) {
                const int sub = (mw >> 1) + 2 * t;
                // (copied to a local first: with the captured array element as the builtin's argument the
                // host pass silently drops this kernel's stub and the library no longer loads)
                const uint32_t vo = voff_l[t];
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    xr, (__attribute__((address_space(3))) void *)(slot + sub * 2048 + half * 1024), 16, vo, 0, 0, 0);
            }
        };
        // write-out of a staged block: this wave stores pixel rows mw*8 .. mw*8+7 through a
        // buffer resource; rows past the range (or a disabled call) get an out-of-range offset
        // and are dropped by the hardware, so every call issues the same number of stores and
        // the vmcnt arithmetic below is uniform
        const rsrc_t yr = make_rsrc(y, (uint32_t)((int64_t)Mtot * KOUT * sizeof(CT)));
        auto store_block = [&](int b, bool enable) {
            const char *stg = out_stage + (b & 1) * kOutBytes;
#pragma unroll
            for (int t = 0; t < kStores; ++t) {
                const int row = mw * 8 + t * (64 / kRowLanes) + lane / kRowLanes;
                const int m = start + b * 32 + row;
                const uint4_t v = *reinterpret_cast<const uint4_t *>(stg + row * kOutPitch + (lane % kRowLanes) * 16);
                const uint32_t off = (uint32_t)m * (uint32_t)(KOUT * sizeof(CT)) + (lane % kRowLanes) * 16;
                __builtin_amdgcn_raw_buffer_store_b128(v, yr, (enable && m < end) ? off : kOutOfRange, 0, 2 /* nt */);
            }
        };
        // Memory operations complete in order, so "block j has landed" is a bound on the number
        // of younger operations.  Steady-state issue order:  ... L(b+1) S(b-3) L(b+2) S(b-2) | barrier b
        // (L = a block's kLoads loads, S = a block's kStores stores); the prologue issues disabled
        // stores so that the same bound holds from the first block on.
        prep_block();
        fire_block(0);
        prep_block();
        fire_block(1);
        store_block(0, false);
        prep_block();
        wait_vmem<kLoads + kStores>();  // block 0 has landed
        wg_barrier();                   // MFMA waves are done with the weight region (slot 2, staging)
        fire_block(2);
        store_block(0, false);
        prep_block();
        for (int b = 0; b < nblocks; ++b) {
            wait_vmem_and_lds<kLoads + 2 * kStores>();  // own part of block b+1 has landed; staging reads are back
            wg_barrier();  // block b+1 complete, slot of block b free, block b-1 staged
            fire_block(b + 3);
            store_block(b - 1, b > 0);
            prep_block();
        }
        wg_barrier();  // the last block is staged
        store_block(nblocks - 1, nblocks > 0);
        wait_vmem_and_lds<0>();
    }
}

// The same division of labour with the input RESIDENT in LDS (stride 1): a workgroup's pixel
// range covers a few output rows of one image, and the input rows under them (range rows +
// R - 1, each with its left and right padding columns, zero-filled by the buffer range check)
// fit the LDS as they are: 9 input rows of 58 pixels for 7 output rows of 56.  They are
// fetched ONCE, in the prologue, instead of once per filter tap as im2col slices, so in the
// steady state the LDS port carries only the operand reads and the output staging (160 KiB
// per 32-pixel block instead of 196), the vector-memory path only the stores, and the MFMA
// waves wait for nothing but their own reads.  A pixel takes 144 bytes (128 of channels + 16
// of padding): with that pitch the 16-byte slots of consecutive pixels fall on 9p mod 16, all
// different within any 16 lanes, so every ds_read_b128 of an operand is conflict free without
// a swizzle, and filter tap (r, s) and the k-substep become an immediate offset
// (s * 144 + ks * 32) on one of R per-lane row addresses.  The patch is filled in linear
// order, 9 chunks of 16 bytes per pixel, the ninth reading out of range.
template <int R, int S, int C, typename CT>
__global__ __launch_bounds__(512) void conv2d_wres_kernel(const uint16_t *__restrict__ x,
                                                          const uint16_t *__restrict__ w, CT *__restrict__ y,
                                                          ConvGeom g, int px_per_wg, int patch_rows)
{
    constexpr int KOUT = 128;               // 4 MFMA waves x 32 channels
    constexpr int KSUB = R * S * C / 16;    // MFMA k-substeps per pixel block
    constexpr int kPerTap = C / 16;         // k-substeps per filter tap
    constexpr int kPix = C * 2 + 16;        // LDS bytes per input pixel
    constexpr int kChunks = kPix / 16;      // 16-byte chunks per pixel, the last one padding
    constexpr int kWeightRegion = 128 * R * S * C;  // prologue: two quarters of every wave's weights
    constexpr int kOutPitch = KOUT * (int)sizeof(CT) + 16;
    constexpr int kOutBytes = 32 * kOutPitch;
    constexpr int kRowLanes = KOUT * (int)sizeof(CT) / 16;  // lanes per pixel row of 16-byte pieces
    constexpr int kStores = 8 * kRowLanes / 64;             // store instructions per memory wave per block (8 rows each)
    constexpr int kWin = 9;                                 // operand window of the MFMA waves
    constexpr int kBar = KSUB - kWin;                       // MFMAs of a block in front of its barrier: behind it the window reads the next block
    constexpr int kFill = 3;                                // patch loads per memory wave and block in the steady state
    static_assert(C == 64 && KSUB % kWin == 0 && 2 * kOutBytes <= kWeightRegion, "layout assumptions");
    static_assert(256 % kChunks == 4 && 256 / kChunks == 28, "the fill's step of 256 chunks is 28 pixels and 4 chunks");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    char *const out_stage = smem;               // (the weight region is free after the first barrier)
    char *const patch = smem + kWeightRegion;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int Mtot = g.N * g.P * g.Q;
    const int wg = gridDim.x % 8 == 0 ? (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
    const int start = wg * px_per_wg, end = min(start + px_per_wg, Mtot);
    const int nblocks = (end - start + 31) / 32;
    // the range lies inside one image (the host checks it): first pixel = (n0, oh0, q0)
    const int n0 = start / (g.P * g.Q), pq0 = start - n0 * (g.P * g.Q);
    const int oh0 = pq0 / g.Q, q0 = pq0 - oh0 * g.Q;
    const int Wv = g.W + 2 * g.pw;  // pixels per patch row; patch row v holds input row oh0 - ph + v
    // chunks per patch row: the Wv pixels and padding up to 9 Q + 32, so that a lane whose pixel
    // wraps to the next output row moves on by a multiple of 256 bytes more than its neighbours:
    // the 16 lanes of a read keep 16 different bank slots across the wrap
    const int row_chunks = kChunks * g.Q + 32;
    // Both kinds of wave execute exactly 2 + nblocks workgroup barriers.
    TL_BEGIN();

    if (wave < 4) {
        // ------------------------------ MFMA waves ------------------------------
        __builtin_amdgcn_s_setprio(2);
        bf16x8_t wf[KSUB];
        load_weight_frags<R, S, C>(wf, smem, w, wave, lane);
        TL_STAMP(wave == 0, 0, 2);
        typedef const __attribute__((address_space(3))) char lds_char_t;
        typedef const __attribute__((address_space(3))) bf16x8_t lds_frag_t;
        lds_char_t *const lds0 = (lds_char_t *)smem;
        // fragment kk = filter tap kk / kPerTap = (r, s), k-substep kk % kPerTap, relative to the
        // lane's address of the pixel under tap (r, 0)
        auto read_frag = [&](const uint32_t (&rowaddr)[R], int kk) {
            const int tap = kk / kPerTap, r = tap / S, sft = tap % S;
            return *(lds_frag_t *)(lds0 + rowaddr[r] + sft * kPix + (kk % kPerTap) * 32);
        };
        // this lane's pixel of block 0: column q0 + lane%32 of the range's first row, or past its end
        // in the second (Q >= 32: one wrap at most); a lane holds channels 8*(lane/32).. of a k-substep
        int ow = q0 + (lane & 31);
        uint32_t pix_addr = (uint32_t)kWeightRegion + (uint32_t)(lane >> 5) * 16u;
        if (ow >= g.Q) {
            ow -= g.Q;
            pix_addr += (uint32_t)(row_chunks * 16);
        }
        pix_addr += (uint32_t)(ow * kPix);
        const uint32_t row_pitch = (uint32_t)(row_chunks * 16), wrap_extra = (uint32_t)(row_chunks * 16 - g.Q * kPix);
        uint32_t cur[R], nxt[R];
        auto rows_of = [&](uint32_t (&a)[R]) {
#pragma unroll
            for (int r = 0; r < R; ++r) a[r] = pix_addr + (uint32_t)r * row_pitch;
        };
        auto next_block = [&]() {  // the lane's pixel 32 further on in the flattened (row, column) order
            ow += 32;
            const bool wrap = ow >= g.Q;
            ow = wrap ? ow - g.Q : ow;
            pix_addr += 32u * kPix + (wrap ? wrap_extra : 0u);
        };
        rows_of(cur);
        // staging position: lane holds channels wave*32 + 8a + 4*(lane/32) + 0..3 of pixel lane%32
        const int stage_wr = (lane & 31) * kOutPitch + (wave * 32 + 4 * (lane >> 5)) * (int)sizeof(CT);
        // bf16: after a permlane32 swap of element groups a and a+1 a lane holds 8 consecutive
        // channels, cg*32 + 8 (a + lane/32) + 0..7, of its pixel: 16-byte writes (8-byte ones at
        // this pitch put lanes p and p+16 on the same banks)
        const int stage_wr16 = (lane & 31) * kOutPitch + (wave * 32 + 8 * (lane >> 5)) * 2;

        wg_barrier();  // the patch is complete (and every wave is done with the weight region)
        TL_STAMP(wave == 0, 0, 3);
        bf16x8_t af[kWin];
#pragma unroll
        for (int kk = 0; kk < kWin; ++kk) af[kk] = read_frag(cur, kk);
        float16_t accs[2];
#pragma unroll
        for (int e = 0; e < 16; ++e) accs[0][e] = accs[1][e] = 0.f;

        // One block: `acc` collects block b, `prev` holds block b-1's results (zeros for b = 0,
        // staged but never written out).  In the shadow of the first MFMAs `prev` is converted
        // and staged, then cleared for block b+1.  The barrier tells the memory waves that it is
        // staged, and the MFMA waves that the patch rows under block b+1 have landed.
        // (blocks come in pairs that swap the two accumulators; the pair is the loop's unit, so that a block
        // boundary carries no loop control)
        auto do_block = [&](int b, auto hc) {
            constexpr int h = decltype(hc)::value;
            float16_t &acc = accs[h];
            float16_t &prev = accs[h ^ 1];
            next_block();
            rows_of(nxt);
            // opaque to the optimiser: folded with the tap offsets they would turn into one address
            // register per read, which does not fit the register budget of two waves per SIMD
#pragma unroll
            for (int r = 0; r < R; ++r) asm volatile("" : "+v"(cur[r]), "+v"(nxt[r]));
            TL_STEP(wave == 0, 0, 8 + b);
            char *stg = out_stage + ((b - 1) & 1) * kOutBytes + stage_wr;
            char *stg16 = out_stage + ((b - 1) & 1) * kOutBytes + stage_wr16;
#pragma unroll
            for (int kk = 0; kk < KSUB; ++kk) {
                if (kk == kBar) {
                    // the staging writes are older than the window's reads: at most kWin LDS
                    // operations outstanding means they are done (lgkmcnt only)
                    __builtin_amdgcn_s_waitcnt(0xC07F | (kWin << 8));
                    wg_barrier();
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[kk], af[kk % kWin], acc, 0, 0, 0);
                af[kk % kWin] = kk + kWin < KSUB ? read_frag(cur, kk + kWin) : read_frag(nxt, kk + kWin - KSUB);
                if constexpr (sizeof(CT) == 4) {
                    if (kk >= 1 && kk < 5) {
                        const int a = kk - 1;
                        *reinterpret_cast<float4_t *>(stg + 8 * a * 4) =
                            float4_t{prev[4 * a], prev[4 * a + 1], prev[4 * a + 2], prev[4 * a + 3]};
                    }
                } else {
                    if (kk == 1 || kk == 3) {
                        const int a = kk - 1;  // element groups a and a + 1
                        const uint32_t x0 = pack_bf16(prev[4 * a], prev[4 * a + 1]), x1 = pack_bf16(prev[4 * a + 2], prev[4 * a + 3]);
                        const uint32_t y0 = pack_bf16(prev[4 * a + 4], prev[4 * a + 5]), y1 = pack_bf16(prev[4 * a + 6], prev[4 * a + 7]);
                        // (lower half-wave: own group a, then the upper lane's; upper: the lower lane's group a+1, then own)
                        const auto s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
                        const auto s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
                        *reinterpret_cast<uint4_t *>(stg16 + 8 * a * 2) = uint4_t{s0[0], s1[0], s0[1], s1[1]};
                    }
                }
                if (kk >= 6 && kk < 10) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) prev[4 * (kk - 6) + e] = 0.f;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) cur[r] = nxt[r];
        };
        int b0 = 0;
        for (; b0 + 1 < nblocks; b0 += 2) {
            do_block(b0, std::integral_constant<int, 0>{});
            do_block(b0 + 1, std::integral_constant<int, 1>{});
        }
        if (b0 < nblocks) do_block(b0, std::integral_constant<int, 0>{});
        // the last block's results
        TL_STAMP(wave == 0, 0, 4);
        const float16_t last = ((nblocks - 1) & 1) ? accs[1] : accs[0];
        stage_acc<CT>(last, out_stage + ((nblocks - 1) & 1) * kOutBytes + stage_wr);
        wait_vmem_and_lds<0>();
        wg_barrier();
        TL_END(wave == 0, 0);
    } else {
        // ------------------------------ memory waves ------------------------------
        const int mw = wave - 4;
        // Patch fill: chunk L of the patch (linear: rows of row_chunks chunks, kChunks per pixel,
        // padding behind the last pixel) is written by lane L % 64 of wave load L / 64; the four
        // waves take the loads in turn, a lane's next chunk is 256 further on.  Padding chunks and
        // pixels outside the image read out of range, i.e. zeros.  Offsets are 32-bit: tensors
        // below 2 GiB (host).
        const rsrc_t xr = make_rsrc(x, (uint32_t)((int64_t)g.N * g.H * g.W * g.C * 2));
        const int nloads = (patch_rows * row_chunks + 63) / 64;
        int rem = mw * 64 + lane, vrow = 0;  // chunk `rem` of patch row `vrow` (the first 256 chunks lie in row 0)
        int next_load = mw;
        auto fire_one = [&]() {
            const int vcol = rem / kChunks, ch = rem - vcol * kChunks;
            const int ih = oh0 - g.ph + vrow, iw = vcol - g.pw;
            const bool ok = ch < kChunks - 1 && vrow < patch_rows && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
            const uint32_t vo = ok ? (uint32_t)(((n0 * g.H + ih) * g.W + iw) * C + ch * 8) * 2u : kOutOfRange;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (__attribute__((address_space(3))) void *)(patch + next_load * 1024), 16,
                                                     vo, 0, 0, 0);
            rem += 256;  // (row_chunks >= 9 * 32 + 32 > 256: one wrap at most)
            if (rem >= row_chunks) {
                rem -= row_chunks;
                ++vrow;
            }
            next_load += 4;
        };
        // Before the first block: the rows under blocks 0 .. 2 (whole rounds of the four waves).
        // From then on kFill loads per wave and block; what block b+1 reads has been issued by
        // the end of step b-2 at the latest (the host checks this schedule for the shape).
        const int rows0 = min(patch_rows, (q0 + 95) / g.Q + R);
        const int loads0 = min((nloads + 3) / 4 * 4, ((rows0 * row_chunks + 63) / 64 + 3) / 4 * 4);
        while (next_load < loads0 && next_load < nloads) fire_one();
        // write-out of a staged block: this wave stores pixel rows mw*8 .. mw*8+7 through a
        // buffer resource; rows past the range get an out-of-range offset and are dropped
        const rsrc_t yr = make_rsrc(y, (uint32_t)((int64_t)Mtot * KOUT * sizeof(CT)));
        auto store_block = [&](int b, bool enable) {
            const char *stg = out_stage + (b & 1) * kOutBytes;
#pragma unroll
            for (int t = 0; t < kStores; ++t) {
                const int row = mw * 8 + t * (64 / kRowLanes) + lane / kRowLanes;
                const int m = start + b * 32 + row;
                const uint4_t v = *reinterpret_cast<const uint4_t *>(stg + row * kOutPitch + (lane % kRowLanes) * 16);
                const uint32_t off = (uint32_t)m * (uint32_t)(KOUT * sizeof(CT)) + (lane % kRowLanes) * 16;
                __builtin_amdgcn_raw_buffer_store_b128(v, yr, (enable && m < end) ? off : kOutOfRange, 0, 2 /* nt */);
            }
        };
        TL_STAMP(wave == 4, 1, 2);
        wait_vmem<0>();  // own part of the first rows has landed
        TL_STAMP(wave == 4, 1, 3);
        wg_barrier();    // the first rows are complete; the MFMA waves are done with the weight region
        TL_STAMP(wave == 4, 1, 4);
        // Memory operations complete in order, so "the loads of step b-2 have landed" is a bound on
        // the number of younger operations: the stores of step b-2 and the loads and stores of
        // step b-1 (every step issues kStores stores, disabled ones while there is nothing to
        // store), so two blocks of stores stay in flight.
        static_assert(kFill + 2 * kStores < 64, "vmcnt is a 6-bit counter");
        int fired = 0;  // loads of the previous step
        for (int b = 0; b < nblocks; ++b) {
            if (fired == kFill) wait_vmem_and_lds<kFill + 2 * kStores>();
            else if (fired == 0) wait_vmem_and_lds<2 * kStores>();
            else wait_vmem_and_lds<kStores>();  // (the step after the one in which the fill ran out)
            wg_barrier();  // block b-1 is staged; the rows under block b+1 are complete
            TL_STEP(wave == 4, 1, 8 + b);
            fired = 0;
#pragma unroll
            for (int t = 0; t < kFill; ++t)
                if (next_load < nloads) {
                    fire_one();
                    ++fired;
                }
            store_block(b - 1, b > 0);
        }
        wg_barrier();  // the last block is staged
        store_block(nblocks - 1, nblocks > 0);
        wait_vmem_and_lds<0>();
        TL_END(wave == 4, 1);
    }
}

// ---- weights-in-registers kernel, 64 output channels per workgroup ---------------------
// The same division of labour once more, with the work cut the other way: a workgroup owns a
// slab of 64 output channels and a pixel range twice as long (K / 64 workgroups share a range).
// It takes in 72 KiB of weights instead of 144, all of them in flight at once and staged in LDS in
// one piece (the 128-channel kernels take theirs in two dependent halves); the price is that every
// input row is fetched by K / 64 workgroups (from the L2 they share: they sit on one XCD).
//   * MFMA wave w holds the weights of channel group w & 1 (32 channels) and computes the pixel
//     blocks of parity w >> 1: in step t the four waves work on blocks 2t and 2t+1, 64 pixels.
//     An operand read serves 32 channels of one wave, so per pixel the LDS carries half the reads
//     of the 128-channel kernels.
//   * The input rows under a range do not fit the LDS any more; they pass through a ring of 8 to 16
//     rows, filled row by row, in groups of 7 pixels, by the memory waves one step ahead of their
//     use.  Wants and free space are counted in whole rows, so a load never writes into a row that
//     is not entirely writable (its 64th lane reaches 16 bytes into the next group of its row).
//   * Every wave first issues one of the rows under the first two steps; the MFMA waves then issue the
//     weight loads (a tap's loads are split between the two waves that need it), and every wave waits
//     for its own loads before the first barrier: behind it every weight is in LDS, and the first two steps
//     run tap-major, reading each tap's weights into registers just ahead of its MFMAs.  (Starting the taps one by one as they
//     land, with a barrier per tap, measured 2.4K cycles slower: every barrier also waited for the
//     memory waves, which were busy issuing the next rows into a saturated memory pipeline.)
//   * Barriers: one when the first rows and the weights are there, one at the end of the first two
//     steps, one after their first results are staged, then one per step, and a last one.
struct WsplitPlan {
    int px = 0;          // pixels per range (a divisor of P*Q); 0: the shape does not fit
    int ranges = 0;      // pixel ranges (workgroups = ranges * K / 64)
    int patch_rows = 0;  // input rows under the longest range
    int row_chunks = 0;  // 16-byte chunks per ring row
    int ring_rows = 0;   // rows of the ring: as many as the LDS holds beside the weight staging, 16 at most
    int rounds = 0;
    size_t lds = 0;
};
constexpr int kWsFill = 5;      // fill loads per memory wave and step
constexpr int kWsStageBytes = 64 * 9 * 64 * 2;  // weight staging: 64 channels x 576 values
constexpr int kWsGroup = 7;     // patch pixels per fill load: 7 x 9 chunks of 16 bytes (+ 1 of the next pixel)

// Fill schedule shared by the kernel and the host's check of it.  A patch row (row v holds input
// row oh0 - pad_h + v, W + 2 pad_w pixels) is fetched in groups of kWsGroup pixels, one load each:
// a lane's pixel within the group and its chunk within the pixel never change, so a load costs the
// memory waves a dozen instructions (they are the critical path of a step: with loads of 64
// consecutive chunks, whose lanes had to divide their position out every time, a step took 1.65K
// cycles against 1.48K without any fill).  Load idx = row idx / groups, group idx % groups; it
// lands in ring row (idx / groups) % ring_rows at pixel kWsGroup * group.
struct WsplitFill {
    int Q, R, patch_rows, groups, ring_rows, q0;
    // rows that hold everything the range's pixels 0 .. px_last need
    __host__ __device__ int rows_through(int px_last) const
    {
        const int r = (q0 + px_last) / Q + R;
        return r < patch_rows ? r : patch_rows;
    }
    // loads wanted once everything through step `t` is to be there; loads that may be issued
    // while step `t_busy` is the oldest one still reading the ring
    __host__ __device__ int wanted(int t) const { return rows_through(64 * t + 63) * groups; }
    __host__ __device__ int writable(int t_busy) const { return ((q0 + 64 * t_busy) / Q + ring_rows) * groups; }
    __host__ __device__ bool fires(int idx, int want, int cap) const { return idx < want && idx < cap && idx < patch_rows * groups; }
};

// n / d for 0 <= n < 2^32 and d >= 1 with the host's m = min(floor(2^32 / d), 2^32 - 1): the high product is the
// quotient or one less (it falls short of n / d by less than n / 2^32 < 1).  A handful of scalar instructions
// where the compiler's division of two run-time values takes about forty, in a prologue whose waves issue one
// instruction every five cycles or so with nothing to hide behind.
struct WsplitMagic {
    uint32_t nslab, pq, q;  // multipliers for K / 64, P * Q and Q
};
static inline uint32_t magic_of(int64_t d) { return d <= 1 ? 0xFFFFFFFFu : (uint32_t)((1ull << 32) / (uint64_t)d); }
__device__ __forceinline__ int fast_div(int n, int d, uint32_t m)
{
    const uint32_t q = __umulhi((uint32_t)n, m);
    return (int)((uint32_t)n - q * (uint32_t)d >= (uint32_t)d ? q + 1 : q);
}

template <int R, int S, int C, typename CT>
__global__ __launch_bounds__(512) void conv2d_wsplit_kernel(const uint16_t *__restrict__ x,
                                                            const uint16_t *__restrict__ w, CT *__restrict__ y,
                                                            ConvGeom g, int px_per_wg, int patch_rows, int row_chunks, int ring_rows,
                                                            WsplitMagic mg)
{
    constexpr int KWG = 64;                 // output channels per workgroup
    constexpr int KSUB = R * S * C / 16;    // MFMA k-substeps per pixel block
    constexpr int kPerTap = C / 16, kTaps = R * S;
    constexpr int kPix = C * 2 + 16;        // LDS bytes per input pixel
    constexpr int kChunks = kPix / 16;
    constexpr int kTapBytes = 32 * C * 2;   // one tap of one channel group in the staging: 4 KiB
    constexpr int kOutPitch = KWG * (int)sizeof(CT) + 16;
    constexpr int kOutBytes = 32 * kOutPitch;               // one staged block
    constexpr int kRowLanes = KWG * (int)sizeof(CT) / 16;   // lanes per pixel row of 16-byte pieces
    constexpr int kStores = 16 * kRowLanes / 64;            // store instructions per memory wave and step (16 pixel rows)
    constexpr int kWin = 9, kBar = KSUB - kWin;
    static_assert(C == 64 && KSUB % kWin == 0 && 4 * kOutBytes <= kWsStageBytes, "layout assumptions");
    static_assert(13 + R <= kBar, "the next step's row addresses are ready before the window reads them");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    char *const out_stage = smem;                  // (the weight staging is free after the tap phase)
    char *const ring = smem + kWsStageBytes;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int Mtot = g.N * g.P * g.Q;
    const int nslab = g.K / KWG;
    const int wg = gridDim.x % 8 == 0 ? (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
    const int range = fast_div(wg, nslab, mg.nslab), slab = wg - range * nslab;
    const int start = range * px_per_wg, end = min(start + px_per_wg, Mtot);
    const int nblocks = (end - start + 31) / 32, nsteps = (nblocks + 1) / 2;
    const int n0 = fast_div(start, g.P * g.Q, mg.pq), pq0 = start - n0 * (g.P * g.Q);
    const int oh0 = fast_div(pq0, g.Q, mg.q), q0 = pq0 - oh0 * g.Q;
    const uint32_t row_pitch = (uint32_t)(row_chunks * 16);
    // Both kinds of wave execute 1 + 1 + (nsteps >= 2) + max(nsteps - 2, 0) + 1 barriers.
    TL_BEGIN();

    // Ring fill: load idx = (patch row, pixel group); a wave takes every `stride`-th.  Per lane: pixel
    // lane / 9 of the group, chunk lane % 9 of the pixel (the ninth is padding: zeros); per load,
    // scalars only.  Lane 63 fetches chunk 0 of the pixel behind the group, the same value that the
    // next group's lane 0 writes there, and the row's last group starts 7 pixels before the row's end
    // (overlapping its neighbour, again with identical values), so every lane of every load writes
    // inside its own ring row whatever the order in which the loads land.
    const rsrc_t xr = make_rsrc(x, (uint32_t)((int64_t)g.N * g.H * g.W * g.C * 2));
    const int Wv = g.W + 2 * g.pw, groups = (Wv + kWsGroup - 1) / kWsGroup;
    const WsplitFill fs{g.Q, R, patch_rows, groups, ring_rows, q0};
    const int lane_px = lane / kChunks, lane_ch = lane - lane_px * kChunks;
    const uint32_t lane_off = (uint32_t)(lane_px * (C * 2) + lane_ch * 16);
    // the wave's next load: its index, group, input row (may lie outside the image), that row's first patch
    // pixel as a pixel index into x (left of the image by the padding), and its ring row's byte offset
    int next_load, fill_grp, fill_ih, fill_rowpix, fill_slot_byte, fill_stride;
    const int ring_bytes = ring_rows * (int)row_pitch;
    auto fill_from = [&](int row, int grp, int stride) {  // (row <= ring_rows)
        next_load = row * groups + grp;
        fill_grp = grp;
        fill_ih = oh0 - g.ph + row;
        fill_rowpix = (n0 * g.H + fill_ih) * g.W - g.pw;
        fill_slot_byte = (row == ring_rows ? 0 : row) * (int)row_pitch;
        fill_stride = stride;
    };
    // (a stride of 4 crosses one row end at most: rows have at least 5 groups)
    auto fire = [&]() {
        const int px0 = min(fill_grp * kWsGroup, Wv - kWsGroup);
        // columns of the image this row offers: none if the row lies above or below it (zeros are written)
        const uint32_t cols = (unsigned)fill_ih < (unsigned)g.H ? (uint32_t)g.W : 0u;
        const uint32_t base = (uint32_t)(fill_rowpix + px0) * (uint32_t)(C * 2);  // (wraps for unused pixels)
        const uint32_t iw = (uint32_t)(px0 - g.pw + lane_px);
        const uint32_t vo = (lane_ch < kChunks - 1 && iw < cols) ? base + lane_off : kOutOfRange;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            xr, (__attribute__((address_space(3))) void *)(ring + fill_slot_byte + px0 * kPix), 16, vo, 0, 0, 0);
        next_load += fill_stride;
        fill_grp += fill_stride;
        if (fill_grp >= groups) {
            fill_grp -= groups;
            ++fill_ih;
            fill_rowpix += g.W;
            fill_slot_byte += (int)row_pitch;
            fill_slot_byte = fill_slot_byte == ring_bytes ? 0 : fill_slot_byte;
        }
    };
    // The rows under steps 0 and 1 (the host has checked that the ring holds them) are the first thing every
    // wave issues, one whole row each (the memory waves rows 0 .. 3, the MFMA waves 4 .. 7, then every eighth):
    // they come from HBM, all 256 workgroups ask at once, and they are what the first MFMA ends up waiting
    // for; the weights behind them come from the L2 and land first.  (With the weights first, the rows dealt out
    // load by load through the general fill below, and the compiler's division sequences in this prologue, the
    // rows had landed 600 cycles later.)
    const int rows_first = fast_div(q0 + 127, g.Q, mg.q) + R < patch_rows ? fast_div(q0 + 127, g.Q, mg.q) + R : patch_rows;
    const int cap0 = ring_rows * groups, want1 = rows_first * groups;
    for (int row = wave >= 4 ? wave - 4 : wave + 4; row < rows_first; row += 8) {
        const int ih = oh0 - g.ph + row;
        const uint32_t cols = (unsigned)ih < (unsigned)g.H ? (uint32_t)g.W : 0u;
        const int rowpix = (n0 * g.H + ih) * g.W - g.pw;
        char *const slot = ring + row * (int)row_pitch;
        for (int grp = 0; grp < groups; ++grp) {
            const int px0 = min(grp * kWsGroup, Wv - kWsGroup);
            const uint32_t base = (uint32_t)(rowpix + px0) * (uint32_t)(C * 2);
            const uint32_t iw = (uint32_t)(px0 - g.pw + lane_px);
            const uint32_t vo = (lane_ch < kChunks - 1 && iw < cols) ? base + lane_off : kOutOfRange;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (__attribute__((address_space(3))) void *)(slot + px0 * kPix), 16, vo,
                                                     0, 0, 0);
        }
    }

    if (wave < 4) {
        // ------------------------------ MFMA waves ------------------------------
        __builtin_amdgcn_s_setprio(2);
        const int grp = wave & 1, par = wave >> 1;
        typedef const __attribute__((address_space(3))) char lds_char_t;
        typedef const __attribute__((address_space(3))) bf16x8_t lds_frag_t;
        lds_char_t *const lds0 = (lds_char_t *)smem;
        // weights of this wave's 32 channels: 18 of its group's 36 loads (the other parity issues the
        // rest), tap by tap; a slot holds 32 channel rows of 128 bytes, chunk c of row ch at position
        // c ^ (ch / 2) % 8 (the 16 rows of a ds_read_b128 phase then fall on 16 different bank slots)
        {
            const rsrc_t wr = make_rsrc(w + (int64_t)(slab * KWG + grp * 32) * (R * S * C), (uint32_t)(32 * R * S * C * 2));
            uint32_t wvo[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = 8 * (2 * par + i) + (lane >> 3);
                wvo[i] = (uint32_t)(row * (R * S * C * 2) + (((lane & 7) ^ ((row >> 1) & 7)) << 4));
            }
#pragma unroll
            for (int t = 0; t < kTaps; ++t)
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const uint32_t vo = wvo[i];
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        wr, (__attribute__((address_space(3))) void *)(smem + (grp * kTaps + t) * kTapBytes + (2 * par + i) * 1024),
                        16, vo, t * (C * 2), 0, 0);
                }
        }
        uint32_t wrd[kPerTap];
#pragma unroll
        for (int j = 0; j < kPerTap; ++j)
            wrd[j] = (uint32_t)(grp * kTaps * kTapBytes + (lane & 31) * (C * 2) + (((2 * j + (lane >> 5)) ^ (((lane & 31) >> 1) & 7)) << 4));
        bf16x8_t wf[KSUB];

        // this lane's pixel: column ow of ring row slot `slot`; a step moves it on by 64 pixels
        int ow = q0 + 32 * par + (lane & 31), slot = 0;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            if (ow >= g.Q) {
                ow -= g.Q;
                ++slot;
            }
        // (Per lane on purpose: a wave-uniform form, two scalar bases per row and a select, replaces most of
        // this vector work by about 60 scalar instructions per step and measured 100-200 cycles per step
        // slower, whether bunched under one MFMA or spread over several.  With the next step's rows simply
        // set equal to this step's, the step is 80 cycles shorter: that is what this arithmetic costs.)
        const uint32_t lane_base = (uint32_t)kWsStageBytes + (uint32_t)(lane >> 5) * 16u;
        auto rows_of = [&](uint32_t (&a)[R]) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                int sl = slot + r;
                sl = sl >= ring_rows ? sl - ring_rows : sl;
                a[r] = lane_base + (uint32_t)sl * row_pitch + (uint32_t)(ow * kPix);
            }
        };
        auto next_step = [&]() {
            ow += 64;
#pragma unroll
            for (int i = 0; i < 2; ++i)
                if (ow >= g.Q) {
                    ow -= g.Q;
                    ++slot;
                }
            slot = slot >= ring_rows ? slot - ring_rows : slot;
        };
        auto read_frag = [&](const uint32_t (&rowaddr)[R], int kk) {
            const int tap = kk / kPerTap, r = tap / S, sft = tap % S;
            return *(lds_frag_t *)(lds0 + rowaddr[r] + sft * kPix + (kk % kPerTap) * 32);
        };
        const int stage_wr = (lane & 31) * kOutPitch + (grp * 32 + 4 * (lane >> 5)) * (int)sizeof(CT);

        uint32_t a0[R], a1[R], cur[R], nxt[R], nxt_px = 0;
        rows_of(a0);
        next_step();
        rows_of(a1);
        bf16x8_t af[kWin];
        float16_t accs[2];
#pragma unroll
        for (int e = 0; e < 16; ++e) accs[0][e] = accs[1][e] = 0.f;

        wait_vmem<0>();  // own weight loads and own first row have landed
        TL_STAMP(wave == 0, 0, 2);
        wg_barrier();    // the weights and the rows under steps 0 and 1 are complete
        TL_STAMP(wave == 0, 0, 3);
        // steps 0 and 1 (step 0 alone if there is no other), tap-major: a tap's weights are read just ahead of its MFMAs
        auto tap_phase = [&](auto nbc) {
            constexpr int NB = decltype(nbc)::value, TOT = KSUB * NB;
            auto frag_at = [&](int p) {  // position p of the MFMA sequence: (tap, step, k-substep)
                const int t = p / (kPerTap * NB), blk = (p / kPerTap) % NB, j = p % kPerTap;
                return read_frag(blk ? a1 : a0, t * kPerTap + j);
            };
#pragma unroll
            for (int p = 0; p < kWin; ++p) af[p] = frag_at(p);
            // the reads of tap t+1's fragments sit in front of tap t's MFMAs
            auto take_tap = [&](auto tc) {
                constexpr int t = decltype(tc)::value;
                if constexpr (t == 0) TL_STAMP(wave == 0, 0, 4);
#pragma unroll
                for (int j = 0; j < kPerTap; ++j) wf[t * kPerTap + j] = *(lds_frag_t *)(lds0 + wrd[j] + t * kTapBytes);
            };
            take_tap(std::integral_constant<int, 0>{});
            static_for<kTaps>([&](auto tc) {
                constexpr int t = decltype(tc)::value;
                if constexpr (t + 1 < kTaps) take_tap(std::integral_constant<int, t + 1>{});
#pragma unroll
                for (int blk = 0; blk < NB; ++blk)
#pragma unroll
                    for (int j = 0; j < kPerTap; ++j) {
                        const int p = (t * NB + blk) * kPerTap + j;
                        accs[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[t * kPerTap + j], af[p % kWin], accs[blk], 0, 0, 0);
                        if (p + kWin < TOT) af[p % kWin] = frag_at(p + kWin);
                        __builtin_amdgcn_sched_barrier(0);
                    }
            });
        };
        if (nsteps >= 2) tap_phase(std::integral_constant<int, 2>{});
        else tap_phase(std::integral_constant<int, 1>{});
        __builtin_amdgcn_s_waitcnt(0xC07F);
        wg_barrier();  // every wave is done with the weight staging; the rows under step 2 have landed
        TL_STAMP(wave == 0, 0, 5);
        // step 2's first operands are asked for before step 0's results are staged: their latency passes behind the
        // conversions and the barrier
        next_step();
        rows_of(cur);
#pragma unroll
        for (int kk = 0; kk < kWin; ++kk) {
            af[kk] = read_frag(cur, kk);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (nsteps >= 2) {
            stage_acc<CT>(accs[0], out_stage + par * kOutBytes + stage_wr);
            __builtin_amdgcn_s_waitcnt(0xC07F);
            wg_barrier();  // step 0 is staged
        }

        // One step: `acc` collects this wave's block of step t (its first MFMA takes a literal zero as C), `prev`
        // holds that of step t-1, which is converted and staged in the shadow of the MFMAs.  The barrier tells
        // the memory waves that it is staged, and the MFMA waves that the rows under step t+1 have landed.
        // (steps come in pairs that swap the two accumulators; the pair is the loop's unit, so a step boundary
        // carries no loop control: the step's first MFMAs are where vector and scalar work is least hidden)
        auto do_step = [&](int t, auto hc) {
            constexpr int h = decltype(hc)::value;
            float16_t &acc = accs[h];
            float16_t &prev = accs[h ^ 1];
            // (opaque to the optimiser: folded with the tap offsets the row addresses would turn into one
            // register per read)
#pragma unroll
            for (int r = 0; r < R; ++r) asm volatile("" : "+v"(cur[r]));
            TL_STEP(wave == 0, 0, 8 + t);
            char *stg = out_stage + ((h ^ 1) * 2 + par) * kOutBytes + stage_wr;  // (t is even where h is 0: step t - 1's buffer)
#pragma unroll
            for (int kk = 0; kk < KSUB; ++kk) {
                // The next step's row addresses, well before their first use and a few instructions per MFMA: vector
                // work hides behind an MFMA only up to the 32 cycles that the MFMA itself takes (all of it in one
                // place, with 64-bit multiply-adds, cost the step 80 cycles).
                if (kk == 8) {
                    ow += 64;
                    asm volatile("" : "+v"(ow));
                }
                if (kk == 9 || kk == 10) {
                    if (ow >= g.Q) {
                        ow -= g.Q;
                        ++slot;
                    }
                    asm volatile("" : "+v"(ow), "+v"(slot));
                }
                if (kk == 11) {
                    slot = slot >= ring_rows ? slot - ring_rows : slot;
                    asm volatile("" : "+v"(slot));
                }
                if (kk == 12) {
                    nxt_px = lane_base + __umul24((uint32_t)ow, (uint32_t)kPix);
                    asm volatile("" : "+v"(nxt_px));
                }
                if (kk >= 13 && kk < 13 + R) {
                    const int r = kk - 13;
                    int sl = slot + r;
                    sl = sl >= ring_rows ? sl - ring_rows : sl;
                    nxt[r] = nxt_px + __umul24((uint32_t)sl, row_pitch);
                    asm volatile("" : "+v"(nxt[r]));
                }
                if (kk == kBar) {
                    __builtin_amdgcn_s_waitcnt(0xC07F | (kWin << 8));
                    wg_barrier();
                }
                if (kk == 0) {
                    float16_t zero;
#pragma unroll
                    for (int e = 0; e < 16; ++e) zero[e] = 0.f;
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[kk], af[kk % kWin], zero, 0, 0, 0);
                } else {
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[kk], af[kk % kWin], acc, 0, 0, 0);
                }
                af[kk % kWin] = kk + kWin < KSUB ? read_frag(cur, kk + kWin) : read_frag(nxt, kk + kWin - KSUB);
                // The previous step's results go to the staging in four pieces, two early and two late in the
                // step (all four right behind the step's first MFMAs cost 30 cycles per step more).  The last one
                // must be complete when the barrier below lets the memory waves read it: LDS operations complete
                // in order and the barrier's wait leaves kWin of them in flight, so kWin operand reads follow it.
                constexpr int kStageAt[4] = {4, 6, 16, 17};
                static_assert(kStageAt[3] + kWin < kBar, "the last staging write is out of the window at the barrier");
                if (kk == kStageAt[0] || kk == kStageAt[1] || kk == kStageAt[2] || kk == kStageAt[3]) {
                    const int a = kk == kStageAt[0] ? 0 : kk == kStageAt[1] ? 1 : kk == kStageAt[2] ? 2 : 3;
                    if constexpr (sizeof(CT) == 4) {
                        *reinterpret_cast<float4_t *>(stg + 8 * a * 4) =
                            float4_t{prev[4 * a], prev[4 * a + 1], prev[4 * a + 2], prev[4 * a + 3]};
                    } else {
                        *reinterpret_cast<uint2_t *>(stg + 8 * a * 2) =
                            uint2_t{pack_bf16(prev[4 * a], prev[4 * a + 1]), pack_bf16(prev[4 * a + 2], prev[4 * a + 3])};
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) cur[r] = nxt[r];
        };
        int t0 = 2;
        for (; t0 + 1 < nsteps; t0 += 2) {
            do_step(t0, std::integral_constant<int, 0>{});
            do_step(t0 + 1, std::integral_constant<int, 1>{});
        }
        if (t0 < nsteps) do_step(t0, std::integral_constant<int, 0>{});
        // the last step's results
        TL_STAMP(wave == 0, 0, 6);
        const float16_t last = ((nsteps - 1) & 1) ? accs[1] : accs[0];
        stage_acc<CT>(last, out_stage + (((nsteps - 1) & 1) * 2 + par) * kOutBytes + stage_wr);
        wait_vmem_and_lds<0>();
        wg_barrier();
        TL_END(wave == 0, 0);
    } else {
        // ------------------------------ memory waves ------------------------------
        const int mw = wave - 4;
        const rsrc_t yr = make_rsrc(y, (uint32_t)((int64_t)Mtot * g.K * sizeof(CT)));
        // write-out of a staged step: this wave stores 16 of its 64 pixel rows (64 channels each)
        auto store_step = [&](int t, bool enable) {
            const char *stg = out_stage + ((t & 1) * 2 + (mw >> 1)) * kOutBytes;
#pragma unroll
            for (int i = 0; i < kStores; ++i) {
                const int row = (mw & 1) * 16 + i * (64 / kRowLanes) + lane / kRowLanes;  // pixel row of block mw >> 1
                const int m = start + t * 64 + (mw >> 1) * 32 + row;
                const uint4_t v = *reinterpret_cast<const uint4_t *>(stg + row * kOutPitch + (lane % kRowLanes) * 16);
                const uint32_t off = (uint32_t)m * (uint32_t)(g.K * sizeof(CT)) + (uint32_t)(slab * KWG * sizeof(CT)) + (lane % kRowLanes) * 16;
                __builtin_amdgcn_raw_buffer_store_b128(v, yr, (enable && m < end) ? off : kOutOfRange, 0, 2 /* nt */);
            }
        };
        TL_STAMP(wave == 4, 1, 2);
        wait_vmem<0>();
        TL_STAMP(wave == 4, 1, 3);
        wg_barrier();  // the rows under steps 0 and 1 are complete
        TL_STAMP(wave == 4, 1, 4);
        // from here on the four memory waves share the fill: first the rows under step 2
        fill_from(rows_first, mw, 4);
        {
            const int rows2 = fast_div(q0 + 191, g.Q, mg.q) + R;
            const int want2 = (rows2 < patch_rows ? rows2 : patch_rows) * groups;
            while (fs.fires(next_load, want2, cap0)) fire();
        }
        wait_vmem_and_lds<0>();
        wg_barrier();  // end of the first two steps: the rows under step 2 are complete; steps 0 and 1 no longer read the ring
        TL_STAMP(wave == 4, 1, 5);
        // Every later iteration issues its fill loads first, then kStores stores: "the loads issued
        // behind the previous barrier have landed" is then vmcnt <= kStores, however many they were.
        // fill_next(): the iteration behind the barrier of step t wants everything through step t + 2
        // and may write the rows below step t's first; both row numbers are stepped on by 64 pixels
        // per call instead of being divided out (first call: t = 1, with step 2 as the oldest reader)
        int want_col = q0 + 64 * 3 + 63, want_row = 0, busy_col = q0 + 64 * 2, busy_row = 0;
        while (want_col >= g.Q) {
            want_col -= g.Q;
            ++want_row;
        }
        while (busy_col >= g.Q) {
            busy_col -= g.Q;
            ++busy_row;
        }
        bool first_fill = true;
        auto fill_next = [&]() {
            const int rows = want_row + R < patch_rows ? want_row + R : patch_rows;
            const int want = rows * groups, cap = (busy_row + ring_rows) * groups;
            for (int i = 0; i < kWsFill && fs.fires(next_load, want, cap); ++i) fire();
            want_col += 64;
#pragma unroll
            for (int i = 0; i < 2; ++i)
                if (want_col >= g.Q) {
                    want_col -= g.Q;
                    ++want_row;
                }
            if (!first_fill) {  // (the first two calls both have step 2 as the oldest reader)
                busy_col += 64;
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    if (busy_col >= g.Q) {
                        busy_col -= g.Q;
                        ++busy_row;
                    }
            }
            first_fill = false;
        };
        if (nsteps >= 2) {
            wg_barrier();  // step 0 is staged
            fill_next();   // wants step 3, step 2 reads
            store_step(0, true);
        }
        for (int t = 2; t < nsteps; ++t) {
            wait_vmem_and_lds<kStores>();
            wg_barrier();  // step t-1 is staged; the rows under step t+1 are complete
            TL_STEP(wave == 4, 1, 8 + t);
            fill_next();   // wants step t + 2; step t may still have operand reads in flight: its rows stay
            store_step(t - 1, true);
        }
        wg_barrier();  // the last step is staged
        store_step(nsteps - 1, nsteps > 0);
        wait_vmem_and_lds<0>();
        TL_END(wave == 4, 1);
    }
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

// Direct convolution for small C: thread = (output pixel, block of KB output channels).
// Each input value is loaded once per thread and multiplied into KB accumulators; the
// block's weights sit in LDS as fp32 [R*S*C][KB], and since every lane reads the same
// address the reads are broadcasts (16 bytes = 4 channels per instruction).
template <int KB, typename T, typename CT>
__global__ __launch_bounds__(256) void conv2d_smallc_kernel(const T *__restrict__ x, const T *__restrict__ w,
                                                            CT *__restrict__ y, ConvGeom g, int64_t npix)
{
    extern __shared__ __attribute__((aligned(16))) float wl[];
    const int taps = g.R * g.S * g.C;
    const int k0 = blockIdx.y * KB;
    for (int i = threadIdx.x; i < taps * KB; i += 256) {
        const int t = i / KB, k = k0 + i % KB;
        wl[i] = k < g.K ? load_xw<T>(w + (int64_t)k * taps + t) : 0.f;
    }
    __syncthreads();
    for (int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x; m < npix; m += (int64_t)gridDim.x * 256) {
        const int q = (int)(m % g.Q), p = (int)((m / g.Q) % g.P);
        const int64_t n = m / ((int64_t)g.P * g.Q);
        float acc[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) acc[kb] = 0.f;
        for (int r = 0; r < g.R; ++r) {
            const int ih = p * g.sh - g.ph + r;
            if (ih < 0 || ih >= g.H) continue;
            for (int sft = 0; sft < g.S; ++sft) {
                const int iw = q * g.sw - g.pw + sft;
                if (iw < 0 || iw >= g.W) continue;
                const T *xp = x + ((n * g.H + ih) * g.W + iw) * g.C;
                const float *wp = wl + (r * g.S + sft) * g.C * KB;
                for (int c = 0; c < g.C; ++c) {
                    const float xv = load_xw<T>(xp + c);
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb) acc[kb] = __builtin_fmaf(xv, wp[c * KB + kb], acc[kb]);
                }
            }
        }
        CT *yp = y + m * g.K + k0;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
            if (k0 + kb < g.K) store_c<CT>(yp + kb, acc[kb]);
    }
}

// ---- few input channels on the matrix cores: one filter row per MFMA -----------------
// With S*C <= 16 the S*C values one pixel needs from one filter row are contiguous in an NHWC
// image row (columns q - pad .. q - pad + S - 1, all channels), so a filter row is a single
// K = 16 step of v_mfma_f32_16x16x16_bf16 (K padded with zero weights): 16 pixels x 16
// output channels take R MFMAs instead of R*S*C*16 vector FMAs per lane group.
// A workgroup of 4 waves owns a tile of 32 output rows x 64 columns of one image (stride 1)
// and one block of 16 output channels.  The 32 + R - 1 input rows of the tile are staged
// once in LDS (aligned dword loads, zero outside the image), in two copies: as loaded, and
// shifted down by one element, so that a lane's 4 values (8 contiguous bytes at a
// 2-byte-aligned position) are two aligned dwords in the copy that matches the parity of its
// position: one ds_read2_b32 instead of four 16-bit reads.  Wave g takes columns
// 16g .. 16g+15 and walks down the staged rows: the operand fragment of input row i feeds
// the R output rows i-R+1 .. i, whose accumulators form a ring of R; the row that has just
// received its last filter row is stored and its accumulator cleared.
// The weights are the MFMA's row operand, so a lane ends up with 4 consecutive output
// channels of one pixel.
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float2_t __attribute__((ext_vector_type(2)));

template <int R, int S, int C, typename CT>
__global__ __launch_bounds__(256) void conv2d_rowmfma_kernel(const uint16_t *__restrict__ x,
                                                             const uint16_t *__restrict__ w, CT *__restrict__ y,
                                                             ConvGeom g, int tiles_w, int tiles_h)
{
    constexpr int TH = 32, TW = 64;
    constexpr int kRows = TH + R - 1;
    // elements per staged row: the last pixel's 16 values plus the odd-start element, even
    constexpr int kPitch = ((TW - 1) * C + 16 + 1 + 1) & ~1;
    static_assert(S * C <= 16 && R <= 8, "one filter row per K = 16 step");
    constexpr int kCopy = kRows * (kPitch / 2);  // dwords of one copy
    __shared__ uint32_t stage32[2 * kCopy];
    // write-out staging, 16 pixels x up to 16 channels per wave: when all K <= 16 channels of a
    // pixel belong to this workgroup, the 16 pixels of a wave's row are one contiguous run of
    // 16*K results in y, written as 16-byte pieces by the first K*sizeof(CT) lanes
    __shared__ __attribute__((aligned(16))) char out_stage[4][16 * 16 * sizeof(CT)];

    const int tid = threadIdx.x, lane = tid & 63, grp = tid >> 6;
    const int tw = blockIdx.x % tiles_w, th = (blockIdx.x / tiles_w) % tiles_h, n = blockIdx.x / (tiles_w * tiles_h);
    const int cb = blockIdx.y;
    const int p0 = th * TH, col0 = tw * TW;
    const int row_elems = g.W * C;                       // even (checked by the host)
    const int e0 = (col0 - g.pw) * C, es = e0 & ~1;      // first element the tile needs; staged from the even one below
    const int delta = e0 - es;
    const uint16_t *ximg = x + (int64_t)n * g.H * row_elems;
    // (all loads of a thread first, then the LDS writes: written as one loop the compiler waits
    // for each load before it issues the next)
    constexpr int kIters = (kCopy + 255) / 256;
    uint32_t sv[kIters];
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int idx = tid + it * 256;
        const int i = idx / (kPitch / 2), d = idx - i * (kPitch / 2);
        const int ih = p0 - g.ph + i, e = es + 2 * d;
        sv[it] = 0;
        if (idx < kCopy && (unsigned)ih < (unsigned)g.H && e >= 0 && e < row_elems)  // e, row_elems even: a pair is inside or outside
            sv[it] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(ximg + (int64_t)ih * row_elems + e));
    }
#pragma unroll
    for (int it = 0; it < kIters; ++it)
        if (tid + it * 256 < kCopy) stage32[tid + it * 256] = sv[it];
    // weights of the 16 channels, zero-padded to [R][16 channels][16 values], through LDS
    __shared__ __attribute__((aligned(8))) uint16_t wst[R * 16 * 16];
    for (int idx = tid; idx < R * 16 * 16; idx += 256) {
        const int k = idx & 15, ch = cb * 16 + ((idx >> 4) & 15), r = idx >> 8;
        wst[idx] = (k < S * C && ch < g.K) ? w[((int64_t)ch * R + r) * (S * C) + k] : (uint16_t)0;
    }
    __syncthreads();
    // this lane's output channel (for the MFMA's row operand): values 4*kg .. 4*kg+3 of filter row r
    const int px = lane & 15, kg = lane >> 4;
    short4_t wf[R];
#pragma unroll
    for (int r = 0; r < R; ++r) wf[r] = *reinterpret_cast<const short4_t *>(wst + (r * 16 + px) * 16 + 4 * kg);
    // second copy: dword d = elements 2d+1, 2d+2 of the row
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int idx = tid + it * 256;
        const int d = idx % (kPitch / 2);
        const uint32_t hi = (idx < kCopy && d + 1 < kPitch / 2) ? stage32[idx + 1] : 0u;
        sv[it] = (sv[it] >> 16) | (hi << 16);
    }
#pragma unroll
    for (int it = 0; it < kIters; ++it)
        if (tid + it * 256 < kCopy) stage32[kCopy + tid + it * 256] = sv[it];
    __syncthreads();

    const int col = col0 + 16 * grp + px;
    const int lb = (16 * grp + px) * C + 4 * kg + delta;  // element offset of this lane's values in a staged row
    const uint32_t *lane_stage = stage32 + (lb & 1) * kCopy + (lb >> 1);
    const int ch0 = cb * 16 + 4 * kg;
    // two results per store when every pair starts at an even element: 32-bit stores of two bf16,
    // 64-bit stores of two floats
    const bool pair_ok = g.K % 2 == 0 && (reinterpret_cast<uintptr_t>(y) & (2 * sizeof(CT) - 1)) == 0;
    const bool run_ok = pair_ok && gridDim.y == 1 && ((int64_t)g.Q * g.K * sizeof(CT)) % 16 == 0 &&
                        (reinterpret_cast<uintptr_t>(y) & 15) == 0 && col0 + 16 * grp + 15 < g.Q;  // uniform per wave
    char *const my_out = out_stage[grp];
    const int run_pieces = g.K * (int)sizeof(CT);  // 16-byte pieces in a wave's run of 16 pixels
    float4_t acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < kRows; ++i) {
        const uint2_t two = {lane_stage[i * (kPitch / 2)], lane_stage[i * (kPitch / 2) + 1]};
        const short4_t bf = __builtin_bit_cast(short4_t, two);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int pl = i - r;  // output row (within the tile) that takes filter row r from input row i
            if (pl >= 0 && pl < TH) acc[pl % R] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(wf[r], bf, acc[pl % R], 0, 0, 0);
        }
        if (i >= R - 1) {
            const int pl = i - (R - 1), p = p0 + pl;
            float4_t &a = acc[pl % R];
            if (run_ok) {
                if (p < g.P) {  // uniform
                    char *o = my_out + (size_t)(px * g.K + ch0) * sizeof(CT);
                    if constexpr (sizeof(CT) == 2) {
                        if (ch0 < g.K) *reinterpret_cast<uint32_t *>(o) = pack_bf16(a[0], a[1]);
                        if (ch0 + 2 < g.K) *reinterpret_cast<uint32_t *>(o + 4) = pack_bf16(a[2], a[3]);
                    } else {
                        if (ch0 < g.K) *reinterpret_cast<float2_t *>(o) = float2_t{a[0], a[1]};
                        if (ch0 + 2 < g.K) *reinterpret_cast<float2_t *>(o + 8) = float2_t{a[2], a[3]};
                    }
                    __builtin_amdgcn_wave_barrier();  // (the wave's LDS operations execute in order)
                    if (lane < run_pieces) {
                        const uint4_t v = *reinterpret_cast<const uint4_t *>(my_out + lane * 16);
                        char *dst = reinterpret_cast<char *>(y + (((int64_t)n * g.P + p) * g.Q + col0 + 16 * grp) * g.K);
                        *reinterpret_cast<uint4_t *>(dst + lane * 16) = v;
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            } else if (p < g.P && col < g.Q) {
                CT *yp = y + (((int64_t)n * g.P + p) * g.Q + col) * g.K + ch0;
                if (pair_ok) {
                    if constexpr (sizeof(CT) == 2) {
                        if (ch0 < g.K) *reinterpret_cast<uint32_t *>(yp) = pack_bf16(a[0], a[1]);
                        if (ch0 + 2 < g.K) *reinterpret_cast<uint32_t *>(yp + 2) = pack_bf16(a[2], a[3]);
                    } else {
                        if (ch0 < g.K) *reinterpret_cast<float2_t *>(yp) = float2_t{a[0], a[1]};
                        if (ch0 + 2 < g.K) *reinterpret_cast<float2_t *>(yp + 2) = float2_t{a[2], a[3]};
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (ch0 + e < g.K) store_c<CT>(yp + e, a[e]);
                }
            }
            a = float4_t{0.f, 0.f, 0.f, 0.f};
        }
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
    static std::atomic<bool> attr_done{false};
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

template <int R, int S, int C, typename CT>
static perf_status launch_conv_wreg(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st)
{
    constexpr int kSlot = (R * S * (C / 32)) * 2048;
    constexpr int kRing = 3 * kSlot + 2 * 32 * (128 * (int)sizeof(CT) + 16);
    constexpr int kWeights = 2 * kSlot + 128 * R * S * C;  // prologue: two quarters of the weights behind ring slots 0 and 1
    constexpr int kLds = kRing > kWeights ? kRing : kWeights;
    static_assert(kLds <= 160 * 1024, "LDS of one CU");
    const int64_t Mtot = (int64_t)g.N * g.P * g.Q;
    int grid = 256;  // one persistent workgroup per CU
    if ((Mtot + 31) / 32 < grid) grid = (int)((Mtot + 31) / 32);
    const int px_per_wg = (int)((Mtot + grid - 1) / grid);
    auto kern = conv2d_wreg_kernel<R, S, C, CT>;
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLds) !=
            hipSuccess)
            return PERF_ERR_LAUNCH;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), kLds, st, (const uint16_t *)x, (const uint16_t *)w, (CT *)y,
                       g, px_per_wg);
    return launch_status();
}

template <int R, int S, int C, typename CT>
static perf_status launch_conv_wres(const void *x, const void *w, void *y, const ConvGeom &g, int px_per_wg,
                                    int patch_rows, size_t lds, hipStream_t st)
{
    const int64_t Mtot = (int64_t)g.N * g.P * g.Q;
    auto kern = conv2d_wres_kernel<R, S, C, CT>;
    // the dynamic-LDS cap is a per-function setting: raised once to the CU's 160 KiB (idempotent, so
    // concurrent first calls are harmless)
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                160 * 1024) != hipSuccess)
            return PERF_ERR_LAUNCH;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(Mtot / px_per_wg)), dim3(512), lds, st, (const uint16_t *)x,
                       (const uint16_t *)w, (CT *)y, g, px_per_wg, patch_rows);
    return launch_status();
}

template <int R, int S, int C, typename CT>
static perf_status launch_conv_wsplit(const void *x, const void *w, void *y, const ConvGeom &g, const WsplitPlan &pl,
                                      hipStream_t st)
{
    auto kern = conv2d_wsplit_kernel<R, S, C, CT>;
    static std::atomic<bool> attr_done{false};  // the dynamic-LDS cap is a per-function, idempotent setting
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                160 * 1024) != hipSuccess)
            return PERF_ERR_LAUNCH;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(pl.ranges * (g.K / 64))), dim3(512), pl.lds, st, (const uint16_t *)x,
                       (const uint16_t *)w, (CT *)y, g, pl.px, pl.patch_rows, pl.row_chunks, pl.ring_rows,
                       WsplitMagic{magic_of(g.K / 64), magic_of((int64_t)g.P * g.Q), magic_of(g.Q)});
    return launch_status();
}

// Launch plan of the 64-channel-slab kernel (stride 1, 3x3): pixel ranges inside one image, the ring
// and the weight staging within the LDS, and the fill schedule replayed for every column a range
// can start in: what step t+1 reads must be issued one iteration before the barrier of step t
// waits for it, within the ring's capacity at that time.
static WsplitPlan plan_wsplit(int64_t N, int64_t P, int64_t Q, int64_t R, int64_t K)
{
    WsplitPlan plan;
    if (K % 64 != 0 || Q < 32) return plan;
    const int64_t nslab = K / 64, Mpix = N * P * Q;
    const int row_chunks = (int)(9 * Q + 32);  // (the 128-channel kernel's pitch: a lane that wraps to the next row keeps its bank slot)
    const int groups = (int)((Q + 2 + kWsGroup - 1) / kWsGroup);  // Q + 2 = W + 2 pad_w patch pixels per row
    const int ring_rows = (int)std::min<int64_t>((160 * 1024 - kWsStageBytes) / (row_chunks * 16), 16);
    const size_t lds = (size_t)kWsStageBytes + (size_t)ring_rows * row_chunks * 16;
    if (ring_rows < 5 || groups < 5) return plan;
    for (int64_t rounds = 1; rounds <= 8 && plan.px == 0; ++rounds) {
        int64_t ranges = 256 * rounds / nslab;
        if (ranges < 1) continue;
        if (ranges > (Mpix + 63) / 64) ranges = (Mpix + 63) / 64;  // at least one step each
        const int64_t px = (Mpix + ranges - 1) / ranges;
        if ((P * Q) % px != 0) continue;
        ranges = Mpix / px;
        const int64_t nb = (px + 31) / 32, nsteps = (nb + 1) / 2, q0max = px % Q == 0 ? 0 : Q - 1;
        const int64_t rows = (q0max + nsteps * 64 - 1) / Q + R;
        bool ok = true;
        for (int64_t q0 = 0; q0 <= q0max && ok; ++q0) {
            const WsplitFill fs{(int)Q, (int)R, (int)rows, groups, ring_rows, (int)q0};
            const int cap0 = ring_rows * groups;
            // the kernel's first phase: the eight waves issue every load below wanted(1), whole rows each (rows
            // that the ring must hold); the four memory waves then go on from the first load beyond it, every
            // fourth each
            const int first = fs.wanted(1);
            ok = first <= cap0;
            int next[4] = {first, first + 1, first + 2, first + 3};
            auto run = [&](int want, int cap, int per_wave) {  // one fill iteration of the four memory waves
                for (int mw = 0; mw < 4; ++mw)
                    for (int i = 0; i < per_wave && fs.fires(next[mw], want, cap); ++i) next[mw] += 4;
            };
            auto covered = [&](int want) {  // every load below `want` has been issued
                const int loads = std::min(want, (int)rows * groups);
                for (int mw = 0; mw < 4; ++mw)
                    if (next[mw] < loads) return false;  // (next[mw]: the first load of wave mw not yet issued)
                return true;
            };
            run(fs.wanted(2), cap0, 1 << 20);
            ok = ok && covered(fs.wanted((int)std::min<int64_t>(2, nsteps - 1)));  // at the end of the first two steps
            if (nsteps >= 2) run(fs.wanted(3), fs.writable(2), kWsFill);
            for (int64_t t = 2; t < nsteps && ok; ++t) {
                ok = covered(fs.wanted((int)std::min<int64_t>(t + 1, nsteps - 1)));  // at the barrier of step t
                run(fs.wanted((int)t + 2), fs.writable((int)t), kWsFill);
            }
        }
        if (ok) {
            plan.px = (int)px;
            plan.ranges = (int)ranges;
            plan.patch_rows = (int)rows;
            plan.row_chunks = row_chunks;
            plan.ring_rows = ring_rows;
            plan.rounds = (int)rounds;
            plan.lds = lds;
        }
    }
    return plan;
}

template <int R, int S, int C, typename CT>
static perf_status launch_conv_rowmfma(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st)
{
    const int tiles_w = (g.Q + 63) / 64, tiles_h = (g.P + 31) / 32;
    hipLaunchKernelGGL((conv2d_rowmfma_kernel<R, S, C, CT>), dim3((unsigned)((int64_t)g.N * tiles_h * tiles_w), (unsigned)((g.K + 15) / 16)),
                       dim3(256), 0, st, (const uint16_t *)x, (const uint16_t *)w, (CT *)y, g, tiles_w, tiles_h);
    return launch_status();
}

// filter shapes with a filter-row-per-MFMA instance
template <typename CT>
static perf_status dispatch_conv_rowmfma(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st)
{
    if (g.R == 5 && g.S == 5 && g.C == 3) return launch_conv_rowmfma<5, 5, 3, CT>(x, w, y, g, st);
    if (g.R == 3 && g.S == 3 && g.C == 3) return launch_conv_rowmfma<3, 3, 3, CT>(x, w, y, g, st);
    if (g.R == 3 && g.S == 3 && g.C == 4) return launch_conv_rowmfma<3, 3, 4, CT>(x, w, y, g, st);
    return PERF_ERR_UNSUPPORTED;
}

constexpr int kSmallcLdsBytes = 48 * 1024;

template <int KB, typename T, typename CT>
static perf_status launch_conv_smallc(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st)
{
    const int64_t npix = (int64_t)g.N * g.P * g.Q;
    int64_t blocks = (npix + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    const unsigned gy = (unsigned)((g.K + KB - 1) / KB);
    const size_t lds = (size_t)g.R * g.S * g.C * KB * sizeof(float);
    hipLaunchKernelGGL((conv2d_smallc_kernel<KB, T, CT>), dim3((unsigned)blocks, gy), dim3(256), lds, st, (const T *)x,
                       (const T *)w, (CT *)y, g, npix);
    return launch_status();
}

template <typename T, typename CT>
static perf_status dispatch_conv_smallc(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st)
{
    if (g.K <= 4) return launch_conv_smallc<4, T, CT>(x, w, y, g, st);
    if (g.K <= 8) return launch_conv_smallc<8, T, CT>(x, w, y, g, st);
    if (g.K <= 12) return launch_conv_smallc<12, T, CT>(x, w, y, g, st);
    return launch_conv_smallc<16, T, CT>(x, w, y, g, st);
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

namespace perf {

enum ConvVariant {
    kConvAuto = 0, kConvWreg = 1, kConvMfma = 2, kConvSmallC = 3, kConvDirect = 4, kConvRowMfma = 5, kConvWres = 6,
    kConvF32Mfma = 7, kConvWsplit = 8
};

// Implicit GEMM on the fp32 matrix instruction: any dtype, stride, padding and channel count.
template <typename T, typename CT>
static perf_status launch_conv_f32mfma(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st)
{
    const int64_t M = (int64_t)g.N * g.P * g.Q, Kred = (int64_t)g.R * g.S * g.C;
    const bool big = ((M + 127) / 128) * ((g.K + 127) / 128) >= 256;
    const int64_t edge = big ? 128 : 64;
    const int64_t gx = (M + edge - 1) / edge, gy = (g.K + edge - 1) / edge;
    if (gx > kMaxGridX || gy > kMaxGridYZ) return PERF_ERR_UNSUPPORTED;
    const ConvRows<T> rows{(const T *)x, g.H, g.W, g.C, g.S, g.sh, g.sw, g.ph, g.pw, g.P, g.Q, M, Kred};
    auto kern = big ? f32mfma_kernel<2, 2, ConvRows<T>, T, CT> : f32mfma_kernel<1, 1, ConvRows<T>, T, CT>;
    // B(k, n) = w[n][k]: the KRSC filter of output channel n is a row of R*S*C values
    hipLaunchKernelGGL(kern, dim3((unsigned)gx, (unsigned)gy, 1), dim3(256), 0, st, rows, (const T *)w, (CT *)y, M,
                       (int64_t)g.K, Kred, (int64_t)1, Kred, (int64_t)g.K, (int64_t)0, (int64_t)0, (int64_t)0, (int64_t)1, 1.0f);
    return launch_status();
}

// variant: kConvAuto = chosen here from the shape; otherwise the caller's choice (perf_conv2d_variant).
static perf_status conv2d_impl(const void *x, const void *w, void *y, int64_t N, int64_t H, int64_t W, int64_t C,
                               int64_t K, int64_t R, int64_t S, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                               int64_t pad_w, perf_dtype xw_dt, perf_dtype y_dt, perf_stream stream, int variant)
{
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
                         ((N * P * Q + 63) / 64) * ((K + 63) / 64) <= kMaxGridX;
    // filter shapes with a weights-in-registers instance
    const bool wreg_ok = mfma_ok && R == 3 && S == 3 && C == 64 && K == 128 && Q >= 32 && N * P * Q * K < (int64_t(1) << 29);
    // ... with the input resident in LDS: stride 1, every workgroup's pixel range inside one image, and
    // the input rows under the longest range (rounded up to whole 32-pixel blocks) fit beside the
    // weight region: rows x (9 Q + 32) chunks of 16 bytes, filled in wave loads of 1 KiB
    int wres_px = 0, wres_rows = 0, wres_rounds = 0;
    size_t wres_lds = 0;
    if (wreg_ok && stride_h == 1 && stride_w == 1) {
        const int64_t Mpix = N * P * Q, blocks = (Mpix + 31) / 32;
        // one workgroup per CU if its rows fit, else the smallest whole number of rounds of 256
        for (int64_t rounds = 1; rounds <= 8 && wres_px == 0; ++rounds) {
            const int64_t grid = blocks < 256 * rounds ? blocks : 256 * rounds;
            const int64_t px = (Mpix + grid - 1) / grid;
            if ((P * Q) % px != 0) continue;
            const int64_t nb = (px + 31) / 32, q0max = px % Q == 0 ? 0 : Q - 1;
            const int64_t rows = (q0max + nb * 32 - 1) / Q + R;
            const int64_t rc = 9 * Q + 32, nloads = (rows * rc + 63) / 64;  // 16-byte chunks per patch row (pixels + padding); wave loads
            const int64_t lds = 128 * R * S * C + nloads * 1024;
            // the kernel's fill schedule: the rows under blocks 0..2 before the first block, then 12
            // loads per block; at the barrier of block b the loads of steps <= b-2 have landed, and
            // the rows under block b+1 must be among them, whatever column q0 the range starts in
            bool fill_ok = true;
            for (int64_t q0 = 0; q0 <= q0max && fill_ok; ++q0) {
                const int64_t rows0 = std::min(rows, (q0 + 95) / Q + R);
                const int64_t loads0 = std::min((nloads + 3) / 4 * 4, ((rows0 * rc + 63) / 64 + 3) / 4 * 4);
                for (int64_t b2 = 0; b2 < nb; ++b2) {
                    const int64_t need = std::min(rows, (q0 + 32 * (b2 + 1) + 31) / Q + R) * rc;
                    const int64_t have = std::min(nloads, loads0 + 12 * std::max<int64_t>(0, b2 - 1)) * 64;
                    if (have < need) fill_ok = false;
                }
            }
            if (lds <= 160 * 1024 && fill_ok) {
                wres_px = (int)px;
                wres_rows = (int)rows;
                wres_rounds = (int)rounds;
                wres_lds = (size_t)lds;
            }
        }
    }
    const bool wres_ok = wres_px > 0;
    // ... 64 output channels per workgroup, input rows through a ring
    WsplitPlan wsplit;
    if (mfma_ok && R == 3 && S == 3 && C == 64 && stride_h == 1 && stride_w == 1 && N * P * Q * K < (int64_t(1) << 29))
        wsplit = plan_wsplit(N, P, Q, R, K);
    const bool wsplit_ok = wsplit.px > 0;
    // few input channels: channel-blocked direct kernel, if a 16-channel block of weights fits its LDS budget
    const bool smallc_ok = R * S * C * 16 * 4 <= kSmallcLdsBytes && (K + 15) / 16 <= kMaxGridYZ;
    // few input channels, one filter row per MFMA K-step: bf16, stride 1, an instantiated filter shape
    const bool rowmfma_ok = xw_dt == PERF_BF16 && stride_h == 1 && stride_w == 1 && (W * C) % 2 == 0 && aligned(x, 4) &&
                            ((R == 5 && S == 5 && C == 3) || (R == 3 && S == 3 && (C == 3 || C == 4))) &&
                            N * H * W * C < (int64_t(1) << 31) && N * ((P + 31) / 32) * ((Q + 63) / 64) <= kMaxGridX &&
                            (K + 15) / 16 <= kMaxGridYZ;
    // fp32 matrix instruction: worth it from 32 output channels on (a 64-wide tile is then at least half used)
    const bool f32mfma_ok = K >= 32 && R * S * C >= 16;
    if (variant == kConvAuto)
        // (the channel-blocked kernel has one thread per pixel: below ~64 workgroups of pixels the
        // thread-per-output kernel has more parallelism and measured faster)
        // (the 64-channel-slab kernel measured ahead of both 128-channel kernels wherever all of them run:
        // 12.3 us against 12.9 on 32x56x56 64 -> 128 with zero operands, 15.4 against 15.8 with random ones,
        // 27.4 against 29.1 on 64x56x56; of those two, the input-resident one pays the weight prologue per
        // workgroup and is ahead of the ring kernel with one or two rounds of workgroups only)
        variant = wsplit_ok                     ? kConvWsplit
                  : (wres_ok && wres_rounds <= 2) ? kConvWres
                  : wreg_ok                     ? kConvWreg
                  : mfma_ok ? kConvMfma
                  : (f32mfma_ok && (xw_dt == PERF_F32 || C >= 32)) ? kConvF32Mfma
                  : (rowmfma_ok && N * P * Q >= 16384)          ? kConvRowMfma
                  : (C < 32 && smallc_ok && N * P * Q >= 16384) ? kConvSmallC
                                                                : kConvDirect;
    else if ((variant == kConvWreg && !wreg_ok) || (variant == kConvMfma && !mfma_ok) ||
             (variant == kConvSmallC && !smallc_ok) || (variant == kConvRowMfma && !rowmfma_ok) ||
             (variant == kConvWres && !wres_ok) || (variant == kConvWsplit && !wsplit_ok) || variant < kConvWreg ||
             variant > kConvWsplit)
        return PERF_ERR_UNSUPPORTED;
    if (variant == kConvWsplit)
        return y_dt == PERF_F32 ? launch_conv_wsplit<3, 3, 64, float>(x, w, y, g, wsplit, st)
                                : launch_conv_wsplit<3, 3, 64, uint16_t>(x, w, y, g, wsplit, st);
    if (variant == kConvF32Mfma) {
        if (xw_dt == PERF_BF16)
            return y_dt == PERF_F32 ? launch_conv_f32mfma<uint16_t, float>(x, w, y, g, st)
                                    : launch_conv_f32mfma<uint16_t, uint16_t>(x, w, y, g, st);
        return y_dt == PERF_F32 ? launch_conv_f32mfma<float, float>(x, w, y, g, st)
                                : launch_conv_f32mfma<float, uint16_t>(x, w, y, g, st);
    }
    if (variant == kConvWres)
        return y_dt == PERF_F32 ? launch_conv_wres<3, 3, 64, float>(x, w, y, g, wres_px, wres_rows, wres_lds, st)
                                : launch_conv_wres<3, 3, 64, uint16_t>(x, w, y, g, wres_px, wres_rows, wres_lds, st);
    if (variant == kConvRowMfma)
        return y_dt == PERF_F32 ? dispatch_conv_rowmfma<float>(x, w, y, g, st) : dispatch_conv_rowmfma<uint16_t>(x, w, y, g, st);
    if (variant == kConvWreg)
        return y_dt == PERF_F32 ? launch_conv_wreg<3, 3, 64, float>(x, w, y, g, st)
                                : launch_conv_wreg<3, 3, 64, uint16_t>(x, w, y, g, st);
    if (variant == kConvMfma) {
        // tile: 128 pixels x 128 channels when that gives every CU two workgroups, else 64 pixels;
        // 64 channels wide when there are no more than 64 (or too few 64 x 128 tiles).  Measured on
        // 8x56x56x64->64 (11.1 -> 7.8 us), 32x56x56x64->64 (27.7 -> 22.7), 8x28x28x128->256 (16.1 -> 11.8);
        // 16x56x56x64->256 keeps the large tile (28 us against 35-38).
        const int64_t Mpix = N * P * Q;
        bool wide = K > 64;
        const bool tall = ((Mpix + 127) / 128) * ((K + (wide ? 127 : 63)) / (wide ? 128 : 64)) >= 512;
        if (!tall && wide && ((Mpix + 63) / 64) * ((K + 127) / 128) < 256) wide = false;
#define PERF_CONV_MFMA(TM, TN)                                                                       \
    (y_dt == PERF_F32 ? launch_conv_mfma<TM, TN, 2, 2, float>(x, w, y, g, st)                        \
                      : launch_conv_mfma<TM, TN, 2, 2, uint16_t>(x, w, y, g, st))
        if (tall) return wide ? PERF_CONV_MFMA(2, 2) : PERF_CONV_MFMA(2, 1);
        return wide ? PERF_CONV_MFMA(1, 2) : PERF_CONV_MFMA(1, 1);
#undef PERF_CONV_MFMA
    }
    if (variant == kConvSmallC) {
        if (xw_dt == PERF_BF16)
            return y_dt == PERF_F32 ? dispatch_conv_smallc<uint16_t, float>(x, w, y, g, st)
                                    : dispatch_conv_smallc<uint16_t, uint16_t>(x, w, y, g, st);
        return y_dt == PERF_F32 ? dispatch_conv_smallc<float, float>(x, w, y, g, st)
                                : dispatch_conv_smallc<float, uint16_t>(x, w, y, g, st);
    }
    if (xw_dt == PERF_BF16)
        return y_dt == PERF_F32 ? launch_conv_direct<uint16_t, float>(x, w, y, g, st)
                                : launch_conv_direct<uint16_t, uint16_t>(x, w, y, g, st);
    return y_dt == PERF_F32 ? launch_conv_direct<float, float>(x, w, y, g, st)
                            : launch_conv_direct<float, uint16_t>(x, w, y, g, st);
}

}  // namespace perf

extern "C" perf_status perf_conv2d(const void *x, const void *w, void *y, int64_t N, int64_t H, int64_t W, int64_t C,
                                   int64_t K, int64_t R, int64_t S, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                                   int64_t pad_w, perf_dtype xw_dt, perf_dtype y_dt, perf_stream stream)
{
    return perf::conv2d_impl(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, xw_dt, y_dt, stream,
                             perf::kConvAuto);
}

extern "C" perf_status perf_conv2d_variant(const void *x, const void *w, void *y, int64_t N, int64_t H, int64_t W,
                                           int64_t C, int64_t K, int64_t R, int64_t S, int64_t stride_h,
                                           int64_t stride_w, int64_t pad_h, int64_t pad_w, perf_dtype xw_dt,
                                           perf_dtype y_dt, int variant, perf_stream stream)
{
    if (variant == perf::kConvAuto) return PERF_ERR_UNSUPPORTED;
    return perf::conv2d_impl(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, xw_dt, y_dt, stream, variant);
}

#ifdef PERF_TIMELINE
// diagnostic build only: the stamps of the last launches of this file's kernels
extern "C" int perf_timeline_fetch_conv(long long *host_out) { return perf::tl_fetch(host_out); }
#endif
