// Device-side helpers shared by the HIP kernels of libany4 (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace any4 {

constexpr int kGroup = 128;   // weights per scale/offset group along K
constexpr int kWave = 64;     // CDNA wavefront

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) {
    return __uint_as_float(bits16 << 16);
}
// high / low half of a packed bf16 pair, widened to fp32
__device__ __forceinline__ float bf16lo_to_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t pair) { return __uint_as_float(pair & 0xFFFF0000u); }

// fp32 -> bf16, round-to-nearest-even; NaN stays a quiet NaN
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// The 16-bit storage type of tables, scales, offsets and activations: bf16, or IEEE fp16 with F16.
// Widening is exact; narrowing rounds to nearest even.
template <bool F16> __device__ __forceinline__ float h16_to_f32(uint32_t bits16) {
    if constexpr (F16) return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
    else return bf16_to_f32(bits16);
}
template <bool F16> __device__ __forceinline__ float h16lo_to_f32(uint32_t pair) {
    if constexpr (F16) return (float)__builtin_bit_cast(_Float16, (uint16_t)(pair & 0xFFFFu));
    else return bf16lo_to_f32(pair);
}
template <bool F16> __device__ __forceinline__ float h16hi_to_f32(uint32_t pair) {
    if constexpr (F16) return (float)__builtin_bit_cast(_Float16, (uint16_t)(pair >> 16));
    else return bf16hi_to_f32(pair);
}
template <bool F16> __device__ __forceinline__ uint32_t f32_to_h16(float f) {
    if constexpr (F16) return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
    else return f32_to_bf16(f);
}

// words per packed row
__host__ __device__ __forceinline__ int64_t row_words(int64_t K, int bits) { return K * bits / 32; }

// Sum over the 64 lanes of a wavefront; every lane gets the total.
// Row-level steps use DPP row rotations, the cross-row steps ds_swizzle / readlane.
__device__ __forceinline__ float wave_sum(float v) {
    // within rows of 16 lanes
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x121 /*row_ror:1*/, 0xF, 0xF, false));
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x122 /*row_ror:2*/, 0xF, 0xF, false));
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x124 /*row_ror:4*/, 0xF, 0xF, false));
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x128 /*row_ror:8*/, 0xF, 0xF, false));
    // across the four rows: swap with lane^16 (ds_swizzle), then lane^32
    v += __uint_as_float(__builtin_amdgcn_ds_swizzle(__float_as_uint(v), 0x401F /*bit-mode xor 0x10*/));
    v += __uint_as_float(__builtin_amdgcn_ds_bpermute(((int)(threadIdx.x & 63) ^ 32) << 2, __float_as_uint(v)));
    return v;
}

}  // namespace any4
