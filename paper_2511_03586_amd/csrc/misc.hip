// Status strings, version, and the two measured ceilings the benchmark prints beside its
// figures: a streaming copy (HBM) and a register-only MFMA loop (matrix cores).
#include "device_utils.h"
#include "host_utils.h"
#include "mfma_tile.h"
#include <type_traits>

namespace perf {

// Each thread moves kCopyUnroll 16-byte vectors per iteration (all loads of an iteration issued
// before its first store).  One vector per thread, i.e. a workgroup per 4 KiB, measured fastest
// for large transfers: 6.47 TB/s on 1 GiB against 6.18 with four per thread (the same at 64 MiB),
// and ahead of every persistent-grid shape of the streaming probe.
constexpr int kCopyUnroll = 1;

__global__ __launch_bounds__(256) void copy_kernel(const uint4_t *__restrict__ src, uint4_t *__restrict__ dst,
                                                   int64_t nvec)
{
    const int64_t stride = (int64_t)gridDim.x * 256 * kCopyUnroll;
    for (int64_t base = (int64_t)blockIdx.x * 256 * kCopyUnroll + threadIdx.x; base < nvec; base += stride) {
        uint4_t v[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u)
            if (base + u * 256 < nvec) v[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u)
            if (base + u * 256 < nvec) __builtin_nontemporal_store(v[u], dst + base + u * 256);
    }
}

// dst 16-byte aligned, src not: a grid of threads, each assembling one 16-byte vector from a source
// it may only assume byte alignment for.
__global__ __launch_bounds__(256) void copy_unaligned_src_kernel(const unsigned char *__restrict__ src,
                                                                 uint4_t *__restrict__ dst, int64_t nvec)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
        uint4_t v;
        __builtin_memcpy(&v, src + i * 16, 16);
        __builtin_nontemporal_store(v, dst + i);
    }
}

__global__ __launch_bounds__(64) void copy_tail_kernel(const unsigned char *__restrict__ src,
                                                       unsigned char *__restrict__ dst, int64_t n)
{
    for (int64_t i = threadIdx.x; i < n; i += 64) dst[i] = src[i];
}

// Streaming probe: the copy kernel's access pattern with its knobs exposed, and its two
// halves on their own.  MODE 0 copy, 1 read only (a per-thread xor keeps the loads alive; one
// dword per workgroup is written to dst), 2 write only.  U = 16-byte vectors per thread and
// iteration (all loads of an iteration are issued before its first store); NTL / NTS =
// non-temporal loads / stores.  The block size is the launch's; with fewer workgroups than
// passes the workgroups loop (persistent grid).
template <int MODE, int U, bool NTL, bool NTS>
__global__ void stream_probe_kernel(const uint4_t *__restrict__ src, uint4_t *__restrict__ dst, int64_t nvec)
{
    const int64_t T = blockDim.x;
    const int64_t stride = (int64_t)gridDim.x * T * U;
    uint4_t keep = {0u, 0u, 0u, 0u};
    for (int64_t base = (int64_t)blockIdx.x * T * U + threadIdx.x; base < nvec; base += stride) {
        uint4_t v[U];
        if constexpr (MODE != 2) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (base + u * T < nvec) v[u] = NTL ? __builtin_nontemporal_load(src + base + u * T) : src[base + u * T];
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = uint4_t{(uint32_t)base, 1u, 2u, (uint32_t)u};
        }
        if constexpr (MODE != 1) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (base + u * T < nvec) {
                    if (NTS) __builtin_nontemporal_store(v[u], dst + base + u * T);
                    else dst[base + u * T] = v[u];
                }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (base + u * T < nvec) keep ^= v[u];
        }
    }
    if constexpr (MODE == 1) {
        // practically never true for real data, but the compiler cannot know: the loads stay
        if ((keep[0] ^ keep[1] ^ keep[2] ^ keep[3]) == 0x9E3779B9u && threadIdx.x == 0)
            reinterpret_cast<uint32_t *>(dst)[blockIdx.x % 4] = keep[0];
    }
}

template <int MODE, int U>
static void launch_stream_probe(const void *src, void *dst, int64_t nvec, int threads, int64_t grid, int policy,
                                hipStream_t st)
{
    const dim3 g((unsigned)grid), b((unsigned)threads);
    const uint4_t *s = (const uint4_t *)src;
    uint4_t *d = (uint4_t *)dst;
    switch (policy & 3) {
    case 0: hipLaunchKernelGGL((stream_probe_kernel<MODE, U, false, false>), g, b, 0, st, s, d, nvec); break;
    case 1: hipLaunchKernelGGL((stream_probe_kernel<MODE, U, true, false>), g, b, 0, st, s, d, nvec); break;
    case 2: hipLaunchKernelGGL((stream_probe_kernel<MODE, U, false, true>), g, b, 0, st, s, d, nvec); break;
    default: hipLaunchKernelGGL((stream_probe_kernel<MODE, U, true, true>), g, b, 0, st, s, d, nvec); break;
    }
}

template <int MODE>
static bool dispatch_stream_probe(const void *src, void *dst, int64_t nvec, int unroll, int threads, int64_t grid,
                                  int policy, hipStream_t st)
{
    switch (unroll) {
    case 1: launch_stream_probe<MODE, 1>(src, dst, nvec, threads, grid, policy, st); return true;
    case 2: launch_stream_probe<MODE, 2>(src, dst, nvec, threads, grid, policy, st); return true;
    case 4: launch_stream_probe<MODE, 4>(src, dst, nvec, threads, grid, policy, st); return true;
    case 8: launch_stream_probe<MODE, 8>(src, dst, nvec, threads, grid, policy, st); return true;
    case 16: launch_stream_probe<MODE, 16>(src, dst, nvec, threads, grid, policy, st); return true;
    }
    return false;
}

// Register-only bf16 MFMA loop: 16 independent 32x32 accumulators per wave (the GEMM's
// 4x4 wave tile), two MFMAs per accumulator and iteration issued back to back as in the
// GEMM main loop, operands constant.  No memory traffic inside the loop, so its rate is
// what the matrix cores sustain at the clock the power management allows.
constexpr int kProbeAcc = 16;
constexpr int kProbeWorkgroups = 256 * 4;

// RANDOM: every accumulator has its own pair of operand registers filled with pseudo-random
// values in [-1, 1), so consecutive MFMAs see different, fully toggling operands, as in a GEMM
// on random data; otherwise one pair of small integers for all.  The clock the power management
// grants depends on that (the same GEMM kernel runs 78 us on zeros and 95-100 us on random data).
template <bool RANDOM>
__global__ __launch_bounds__(256) void mfma_probe_kernel(float *__restrict__ sink, int64_t iters)
{
    const int lane = threadIdx.x & 63;
    constexpr int kSets = RANDOM ? kProbeAcc : 1;
    bf16x8_t as[kSets], bs[kSets];
#pragma unroll
    for (int i = 0; i < kSets; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (RANDOM) {
                uint32_t h = (uint32_t)(threadIdx.x * 131 + i * 17 + e) * 2654435761u;
                h ^= h >> 15;
                h *= 2246822519u;
                h ^= h >> 13;
                as[i][e] = (__bf16)((float)(h & 0xFFFF) * (1.0f / 32768.0f) - 1.0f);
                bs[i][e] = (__bf16)((float)(h >> 16) * (1.0f / 32768.0f) - 1.0f);
            } else {
                as[i][e] = (__bf16)(float)((lane + e) & 3);
                bs[i][e] = (__bf16)(float)((lane ^ e) & 1);
            }
        }
    float16_t acc[kProbeAcc];
#pragma unroll
    for (int i = 0; i < kProbeAcc; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kProbeAcc; ++i) {
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as[i % kSets], bs[i % kSets], acc[i], 0, 0, 0);
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bs[i % kSets], as[i % kSets], acc[i], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < kProbeAcc; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    if (lane == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = s;
}

// LDS read probes (256 workgroups, one per CU; every wave reads conflict-free, lane l at 16 l or, for
// the operand pattern, pixel l % 32 at a pitch of 144 bytes plus 16 (l / 32) bytes):
//   MFMA = false: 16 reads of BYTES per lane in flight, then all consumed; cycles of the slowest wave
//                 of workgroup 0 for iters * 16 reads, from which the caller derives bytes per clock and CU.
//   MFMA = true:  the convolution kernels' inner pattern, one v_mfma_f32_32x32x16_bf16 and one
//                 ds_read_b128 of the operand needed nine MFMAs later, 36 per iteration; cycles of
//                 the slowest wave for iters * 36 MFMAs (32 each is the matrix core's own time).
template <int BYTES, bool MFMA, bool VALU = false>
__global__ __launch_bounds__(1024) void lds_probe_kernel(long long *__restrict__ cycles, float *__restrict__ sink, int64_t iters)
{
    __shared__ __attribute__((aligned(1024))) char smem[65536];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x) reinterpret_cast<float *>(smem)[i] = 0.f;
    __syncthreads();
    float keep = 0.f;
    long long c0 = 0, c1 = 0;
    if constexpr (MFMA) {
        typedef const __attribute__((address_space(3))) bf16x8_t lds_frag_t;
        typedef const __attribute__((address_space(3))) char lds_char_t;
        lds_char_t *base = (lds_char_t *)smem;
        const uint32_t addr = (uint32_t)((wave & 3) * 8192 + (lane & 31) * 144 + (lane >> 5) * 16);
        bf16x8_t wgt, af[9];
#pragma unroll
        for (int e = 0; e < 8; ++e) wgt[e] = (__bf16)1.0f;
#pragma unroll
        for (int i = 0; i < 9; ++i) {
            af[i] = *(lds_frag_t *)(base + addr + i * 32);
            __builtin_amdgcn_sched_barrier(0);
        }
        float16_t acc;
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] = 0.f;
        uint32_t x = (uint32_t)lane;
        c0 = __builtin_readcyclecounter();
        for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
            for (int kk = 0; kk < 36; ++kk) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wgt, af[kk % 9], acc, 0, 0, 0);
                af[kk % 9] = *(lds_frag_t *)(base + addr + ((kk + 9) % 16) * 32);
                if (VALU && kk >= 12 && kk < 16) {  // 5 dependent 32-bit multiply-adds behind each of 4 MFMAs
#pragma unroll
                    for (int r = 0; r < 5; ++r) {
                        x = x * 1664525u + 1013904223u;
                        asm volatile("" : "+v"(x));
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        c1 = __builtin_readcyclecounter();
#pragma unroll
        for (int e = 0; e < 16; ++e) keep += acc[e];
        if (VALU && x == 77u) keep = 12345.678f;  // (x is live; whether this ever holds is irrelevant to the timing)
    } else {
        typedef float vecn_t __attribute__((ext_vector_type(BYTES == 4 ? 2 : BYTES / 4)));
        using vec_t = std::conditional_t<BYTES == 4, float, vecn_t>;
        const char *base = smem + (wave & 3) * 16384 + lane * BYTES;
        c0 = __builtin_readcyclecounter();
        for (int64_t it = 0; it < iters; ++it) {
            vec_t v[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) v[k] = *reinterpret_cast<const vec_t *>(base + k * 64 * BYTES);
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                asm volatile("" : "+v"(v[k]));
                if constexpr (BYTES == 4) keep += v[k];
                else keep += v[k][0];
            }
        }
        c1 = __builtin_readcyclecounter();
    }
    if (blockIdx.x == 0 && lane == 0) atomicMax(reinterpret_cast<unsigned long long *>(cycles), (unsigned long long)(c1 - c0));
    if (keep == 12345.678f) sink[0] = keep;  // (never true: the reads stay live)
}

// L2 -> CU feed probe: every workgroup streams 1 KiB wave loads from a window of `span` bytes (its own, or one all
// workgroups share), eight per wavefront and iteration with another eight in flight, window offset
// ((it * 8 + u) * waves + wave) KiB mod span, so a window larger than the L1 is served by the L2.
//   MODE 0: buffer_load ... lds, lane i -> bytes 16 i of the KiB      MODE 1: load to registers, then ds_write_b128
//   MODE 2: load to registers only                                     MODE 3: buffer_load ... lds in the slab
//   convolution's row pattern (7 pixels x 8 lanes of 16 bytes, every ninth lane out of range: zeros)
template <int MODE>
__global__ __launch_bounds__(512) void feed_probe_kernel(const char *__restrict__ src, long long *__restrict__ cycles,
                                                         float *__restrict__ sink, int iters, int shared, uint32_t span)
{
    __shared__ __attribute__((aligned(1024))) char smem[65536];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = blockDim.x >> 6;
    const rsrc_t r = make_rsrc(src + (shared ? 0 : (size_t)blockIdx.x * span), span);
    float keep = 0.f;
    __syncthreads();
    const long long c0 = __builtin_readcyclecounter();
    if constexpr (MODE == 0 || MODE == 3) {
        uint32_t vo = (uint32_t)(lane * 16);
        if constexpr (MODE == 3) vo = lane % 9 < 8 ? (uint32_t)(lane / 9 * 128 + lane % 9 * 16) : kOutOfRange;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t kib = (uint32_t)(((it * 8 + u) * nw + wave) * 1024);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void *)(smem + (kib & 65535)), 16, vo,
                                                         kib & (span - 1), 0, 0);
            }
            wait_vmem<8>();
        }
        wait_vmem<0>();
    } else {
        uint4_t a[8], b[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            a[u] = __builtin_amdgcn_raw_buffer_load_b128(r, (uint32_t)(lane * 16), (uint32_t)(((u * nw + wave) * 1024) & (span - 1)), 0);
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
                b[u] = __builtin_amdgcn_raw_buffer_load_b128(r, (uint32_t)(lane * 16),
                                                             (uint32_t)((((it + 1) * 8 + u) * nw + wave) * 1024) & (span - 1), 0);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if constexpr (MODE == 1) {
                    *reinterpret_cast<uint4_t *>(smem + (((u * nw + wave) * 1024) & 65535) + lane * 16) = a[u];
                } else {
                    asm volatile("" : "+v"(a[u]));
                    keep += __builtin_bit_cast(float, a[u][0]);
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] = b[u];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) keep += __builtin_bit_cast(float, a[u][1]);
    }
    __syncthreads();
    const long long c1 = __builtin_readcyclecounter();
    if (MODE != 2) keep += reinterpret_cast<float *>(smem)[threadIdx.x];
    if (blockIdx.x == 0 && lane == 0) atomicMax(reinterpret_cast<unsigned long long *>(cycles), (unsigned long long)(c1 - c0));
    if (keep == 12345.678f) sink[0] = keep;  // (never true for the zero-filled or finite inputs a caller passes: the loads stay live)
}

}  // namespace perf

static perf_status mfma_probe(float *sink, int64_t iters, bool random, perf_stream stream)
{
    using namespace perf;
    if (!sink) return PERF_ERR_NULL;
    if (iters < 1 || iters > (int64_t(1) << 24)) return PERF_ERR_SHAPE;
    if (!aligned(sink, 4)) return PERF_ERR_ALIGN;
    auto kern = random ? mfma_probe_kernel<true> : mfma_probe_kernel<false>;
    hipLaunchKernelGGL(kern, dim3(kProbeWorkgroups), dim3(256), 0, static_cast<hipStream_t>(stream), sink, iters);
    return launch_status();
}

extern "C" perf_status perf_mfma_probe(float *sink, int64_t iters, perf_stream stream)
{
    return mfma_probe(sink, iters, false, stream);
}

extern "C" perf_status perf_mfma_probe_random(float *sink, int64_t iters, perf_stream stream)
{
    return mfma_probe(sink, iters, true, stream);
}

extern "C" perf_status perf_lds_probe(long long *cycles, float *sink, int waves, int bytes_per_lane, int with_mfma,
                                      int64_t iters, perf_stream stream)
{
    using namespace perf;
    if (!cycles || !sink) return PERF_ERR_NULL;
    if ((waves != 4 && waves != 8 && waves != 16) || (bytes_per_lane != 4 && bytes_per_lane != 8 && bytes_per_lane != 16) ||
        iters < 1 || iters > (int64_t(1) << 24))
        return PERF_ERR_SHAPE;
    if (with_mfma < 0 || with_mfma > 2) return PERF_ERR_SHAPE;
    if (with_mfma && bytes_per_lane != 16) return PERF_ERR_UNSUPPORTED;
    if (!aligned(cycles, 8) || !aligned(sink, 4)) return PERF_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid(256), block(64 * waves);
    if (with_mfma == 2) hipLaunchKernelGGL((lds_probe_kernel<16, true, true>), grid, block, 0, st, cycles, sink, iters);
    else if (with_mfma) hipLaunchKernelGGL((lds_probe_kernel<16, true>), grid, block, 0, st, cycles, sink, iters);
    else if (bytes_per_lane == 16) hipLaunchKernelGGL((lds_probe_kernel<16, false>), grid, block, 0, st, cycles, sink, iters);
    else if (bytes_per_lane == 8) hipLaunchKernelGGL((lds_probe_kernel<8, false>), grid, block, 0, st, cycles, sink, iters);
    else hipLaunchKernelGGL((lds_probe_kernel<4, false>), grid, block, 0, st, cycles, sink, iters);
    return launch_status();
}

extern "C" perf_status perf_feed_probe(const void *src, int64_t src_bytes, long long *cycles, float *sink, int waves, int mode,
                                       int shared, int64_t span, int64_t iters, perf_stream stream)
{
    using namespace perf;
    if (!src || !cycles || !sink) return PERF_ERR_NULL;
    if ((waves != 4 && waves != 8) || mode < 0 || mode > 3 || (shared != 0 && shared != 1) || iters < 1 || iters > (1 << 14))
        return PERF_ERR_SHAPE;  // (the byte offset (iters + 1) * 8 * waves KiB stays below 2^31)
    if (span < 1024 || span > (1 << 30) || (span & (span - 1)) != 0) return PERF_ERR_SHAPE;
    if (src_bytes < (shared ? span : 256 * span)) return PERF_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(cycles, 8) || !aligned(sink, 4)) return PERF_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid(256), block(64 * waves);
    const char *s = static_cast<const char *>(src);
    if (mode == 0) hipLaunchKernelGGL(feed_probe_kernel<0>, grid, block, 0, st, s, cycles, sink, (int)iters, shared, (uint32_t)span);
    else if (mode == 1) hipLaunchKernelGGL(feed_probe_kernel<1>, grid, block, 0, st, s, cycles, sink, (int)iters, shared, (uint32_t)span);
    else if (mode == 2) hipLaunchKernelGGL(feed_probe_kernel<2>, grid, block, 0, st, s, cycles, sink, (int)iters, shared, (uint32_t)span);
    else hipLaunchKernelGGL(feed_probe_kernel<3>, grid, block, 0, st, s, cycles, sink, (int)iters, shared, (uint32_t)span);
    return launch_status();
}

extern "C" perf_status perf_copy(const void *src, void *dst, int64_t bytes, perf_stream stream)
{
    using namespace perf;
    if (!src || !dst) return PERF_ERR_NULL;
    if (bytes < 0) return PERF_ERR_SHAPE;
    if (bytes == 0) return PERF_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned char *sp = static_cast<const unsigned char *>(src);
    unsigned char *dp = static_cast<unsigned char *>(dst);
    // head: the bytes in front of dst's first 16-byte boundary (a few, one small workgroup)
    int64_t head = (int64_t)((16 - (reinterpret_cast<uintptr_t>(dp) & 15)) & 15);
    if (head > bytes) head = bytes;
    if (head > 0) hipLaunchKernelGGL(copy_tail_kernel, dim3(1), dim3(64), 0, st, sp, dp, head);
    sp += head;
    dp += head;
    const int64_t nvec = (bytes - head) / 16;
    if (nvec > 0) {
        if (aligned(sp, 16)) {
            int64_t blocks = (nvec + 256 * kCopyUnroll - 1) / (256 * kCopyUnroll);
            if (blocks > 256 * 1024) blocks = 256 * 1024;  // one pass per workgroup measured faster than a long grid-stride loop
            hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const uint4_t *)sp, (uint4_t *)dp, nvec);
        } else {
            int64_t blocks = (nvec + 255) / 256;
            if (blocks > 256 * 64) blocks = 256 * 64;
            hipLaunchKernelGGL(copy_unaligned_src_kernel, dim3((unsigned)blocks), dim3(256), 0, st, sp, (uint4_t *)dp, nvec);
        }
    }
    const int64_t done = head + nvec * 16;
    if (done < bytes)
        hipLaunchKernelGGL(copy_tail_kernel, dim3(1), dim3(64), 0, st, sp + nvec * 16, dp + nvec * 16, bytes - done);
    return launch_status();
}

extern "C" perf_status perf_stream_probe(const void *src, void *dst, int64_t bytes, int mode, int unroll, int threads,
                                         int64_t grid, int policy, perf_stream stream)
{
    using namespace perf;
    if (!src || !dst) return PERF_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0 || mode < 0 || mode > 2 || policy < 0 || policy > 3 || grid < 0 ||
        grid > kMaxGridX || (threads != 64 && threads != 128 && threads != 256 && threads != 512 && threads != 1024))
        return PERF_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(dst, 16)) return PERF_ERR_ALIGN;
    if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8 && unroll != 16) return PERF_ERR_UNSUPPORTED;
    const int64_t nvec = bytes / 16;
    int64_t passes = (nvec + (int64_t)threads * unroll - 1) / ((int64_t)threads * unroll);
    if (passes > kMaxGridX) return PERF_ERR_SHAPE;
    if (grid == 0 || grid > passes) grid = passes;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (mode == 0) dispatch_stream_probe<0>(src, dst, nvec, unroll, threads, grid, policy, st);
    else if (mode == 1) dispatch_stream_probe<1>(src, dst, nvec, unroll, threads, grid, policy, st);
    else dispatch_stream_probe<2>(src, dst, nvec, unroll, threads, grid, policy, st);
    return launch_status();
}

extern "C" const char *perf_status_string(perf_status s)
{
    switch (s) {
    case PERF_OK: return "ok";
    case PERF_ERR_NULL: return "null pointer";
    case PERF_ERR_SHAPE: return "bad shape, leading dimension, stride or padding";
    case PERF_ERR_DTYPE: return "bad dtype";
    case PERF_ERR_LAYOUT: return "bad layout";
    case PERF_ERR_ALIGN: return "misaligned pointer";
    case PERF_ERR_UNSUPPORTED: return "unsupported combination";
    case PERF_ERR_LAUNCH: return "HIP launch error";
    }
    return "unknown status";
}

extern "C" int perf_version(void) { return 100; }
