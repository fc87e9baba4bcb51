// Cycle-counter timeline of a kernel's phases: a diagnostic build of the same kernels, compiled
// in only with -DPERF_TIMELINE=1 (phase stamps) or -DPERF_TIMELINE=2 (plus one stamp per step of
// the main loop).  Without the macro every TL_* line below is empty and the kernels are the
// product's.  One lane of one wave per role writes "cycles since the workgroup started" into
// tl_buf[workgroup][role][slot]; slot 0 is the last stamp's cycle count, slot 1 the constant
// 100 MHz clock over the same span (their ratio is the shader clock the kernel ran at).
// Reading the cycle counter waits for the wave's outstanding LDS reads (it returns through
// the same counter), so a stamp costs the wave its read pipeline once: level 1 stamps only
// between phases, level 2 shows the steps' relative weights, not their undisturbed length.
// The extra global stores are younger than the loads the kernels' counted waits ask about, so
// those waits stay sufficient.
#pragma once
#include <hip/hip_runtime.h>

#ifdef PERF_TIMELINE
namespace perf {
constexpr int kTlGroups = 256, kTlRoles = 2, kTlSlots = 64;
static __device__ long long tl_buf[kTlGroups][kTlRoles][kTlSlots];
struct TlClock {
    long long c0, r0;
};
__device__ __forceinline__ TlClock tl_begin() { return TlClock{(long long)__builtin_readcyclecounter(), (long long)__builtin_amdgcn_s_memrealtime()}; }
__device__ __forceinline__ void tl_stamp(const TlClock &k, bool who, int role, int slot)
{
    if (who && (threadIdx.x & 63) == 0 && blockIdx.x < kTlGroups && slot >= 2 && slot < kTlSlots)
        tl_buf[blockIdx.x][role][slot] = (long long)__builtin_readcyclecounter() - k.c0;
}
__device__ __forceinline__ void tl_end(const TlClock &k, bool who, int role)
{
    if (who && (threadIdx.x & 63) == 0 && blockIdx.x < kTlGroups) {
        tl_buf[blockIdx.x][role][0] = (long long)__builtin_readcyclecounter() - k.c0;
        tl_buf[blockIdx.x][role][1] = (long long)__builtin_amdgcn_s_memrealtime() - k.r0;
    }
}
// host: copy this translation unit's buffer out (kTlGroups * kTlRoles * kTlSlots values) and clear it
static inline int tl_fetch(long long *host_out)
{
    if (hipDeviceSynchronize() != hipSuccess) return 1;
    if (hipMemcpyFromSymbol(host_out, HIP_SYMBOL(tl_buf), sizeof(long long) * kTlGroups * kTlRoles * kTlSlots) != hipSuccess) return 2;
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(tl_buf)) != hipSuccess) return 3;
    return hipMemset(p, 0, sizeof(long long) * kTlGroups * kTlRoles * kTlSlots) == hipSuccess ? 0 : 4;
}
}  // namespace perf
#define TL_BEGIN() const perf::TlClock tl_clk = perf::tl_begin()
#define TL_STAMP(who, role, slot) perf::tl_stamp(tl_clk, (who), (role), (slot))
#define TL_END(who, role) perf::tl_end(tl_clk, (who), (role))
#define TL_DRAIN() __builtin_amdgcn_s_waitcnt(0x0F70) /* vmcnt(0): the stamp that follows is "stores complete" */
#if PERF_TIMELINE >= 2
#define TL_STEP(who, role, slot) perf::tl_stamp(tl_clk, (who), (role), (slot))
#else
#define TL_STEP(who, role, slot) do {} while (0)
#endif
#else
#define TL_BEGIN() do {} while (0)
#define TL_STAMP(who, role, slot) do {} while (0)
#define TL_END(who, role) do {} while (0)
#define TL_DRAIN() do {} while (0)
#define TL_STEP(who, role, slot) do {} while (0)
#endif
