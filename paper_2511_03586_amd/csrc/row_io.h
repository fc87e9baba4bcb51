// Element access shared by the row-wise streaming kernels (LayerNorm, RMS norm, means):
// 16-byte chunks of fp32 or bf16 unpacked to fp32 registers, and packed stores.
#pragma once
#include "device_utils.h"

namespace perf {

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kPerChunk = 4;  // elements in one 16-byte load
    __device__ static __forceinline__ void unpack(uint4_t raw, float *v)
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t bits = raw[e];  // a bit cast must not be applied to a vector element directly
            v[e] = __builtin_bit_cast(float, bits);
        }
    }
    __device__ static __forceinline__ float load1(const float *p) { return *p; }
    __device__ static __forceinline__ void store1(float *p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {  // bf16 bit patterns
    static constexpr int kPerChunk = 8;
    __device__ static __forceinline__ void unpack(uint4_t raw, float *v)
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[2 * e] = bf16_lo(raw[e]);
            v[2 * e + 1] = bf16_hi(raw[e]);
        }
    }
    __device__ static __forceinline__ float load1(const uint16_t *p) { return bf16_to_f32(*p); }
    __device__ static __forceinline__ void store1(uint16_t *p, float v) { *p = f32_to_bf16(v); }
};

// Store E fp32 values as YT starting at y (16-byte aligned for the group).
template <typename YT, int E>
__device__ __forceinline__ void store_chunk(YT *y, const float *v)
{
    if constexpr (sizeof(YT) == 4) {
#pragma unroll
        for (int q = 0; q < E / 4; ++q)
            __builtin_nontemporal_store(float4_t{v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]},
                                        reinterpret_cast<float4_t *>(y) + q);
    } else if constexpr (E == 8) {
        uint4_t o = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
        __builtin_nontemporal_store(o, reinterpret_cast<uint4_t *>(y));
    } else {
        uint2_t o = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        __builtin_nontemporal_store(o, reinterpret_cast<uint2_t *>(y));
    }
}

}  // namespace perf
