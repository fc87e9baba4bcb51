// Device-side helpers for gfx950 (wave64): DPP / permlane wave reductions, bf16
// conversion, 128-bit vector types. HIP kernels only; nothing here is shared with the
// CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace perf {

constexpr int kWave = 64;

typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

// ---- bf16 <-> fp32 -------------------------------------------------------------
// A bf16 is the top half of an fp32: widening is a shift, exact.
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __builtin_bit_cast(float, packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __builtin_bit_cast(float, packed & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }

// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    bf16x2_t v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}

// ---- wave64 all-reduce ---------------------------------------------------------
// Butterfly over 64 lanes without touching LDS: quad_perm (xor 1, xor 2), row_half_mirror
// and row_mirror (lanes 4 and 8 apart once quads / octets are uniform), then the gfx950
// permlane16_swap / permlane32_swap, which exchange odd rows of 16 (resp. the upper
// half-wave) of the first operand with even rows (the lower half-wave) of the second.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    int b = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(b, b, CTRL, 0xF, 0xF, false));
}

struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return __builtin_fmaxf(a, b); } };
struct OpMin { __device__ __forceinline__ float operator()(float a, float b) const { return __builtin_fminf(a, b); } };
struct OpSum { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };

// permlane16_swap / permlane32_swap of a value with itself: returns in (a, b) the two
// registers the instruction leaves, i.e. for permlane16 a = rows (0,0,2,2) and
// b = rows (1,1,3,3) of v; for permlane32 a = (low half, low half), b = (high, high).
// The two results are copied to scalars before the bit cast: a bit cast applied to a
// vector-element expression reads element 0 whatever the index.
__device__ __forceinline__ void swap16(float v, float &a, float &b)
{
    const unsigned u = __builtin_bit_cast(unsigned, v);
    auto p = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const unsigned p0 = p[0], p1 = p[1];
    a = __builtin_bit_cast(float, p0);
    b = __builtin_bit_cast(float, p1);
}
__device__ __forceinline__ void swap32(float v, float &a, float &b)
{
    const unsigned u = __builtin_bit_cast(unsigned, v);
    auto p = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned p0 = p[0], p1 = p[1];
    a = __builtin_bit_cast(float, p0);
    b = __builtin_bit_cast(float, p1);
}

template <typename Op>
__device__ __forceinline__ float wave_allreduce(float v, Op op)
{
    v = op(v, dpp_move<0xB1>(v));   // quad_perm [1,0,3,2]
    v = op(v, dpp_move<0x4E>(v));   // quad_perm [2,3,0,1]
    v = op(v, dpp_move<0x141>(v));  // row_half_mirror
    v = op(v, dpp_move<0x140>(v));  // row_mirror
    float a, b;
    swap16(v, a, b);
    v = op(a, b);
    swap32(v, a, b);
    v = op(a, b);
    return v;
}

// All-reduce over each half of the wave (lanes 0-31 and 32-63 separately).
template <typename Op>
__device__ __forceinline__ float half_allreduce(float v, Op op)
{
    v = op(v, dpp_move<0xB1>(v));   // quad_perm [1,0,3,2]
    v = op(v, dpp_move<0x4E>(v));   // quad_perm [2,3,0,1]
    v = op(v, dpp_move<0x141>(v));  // row_half_mirror
    v = op(v, dpp_move<0x140>(v));  // row_mirror
    float a, b;
    swap16(v, a, b);
    return op(a, b);
}

}  // namespace perf
