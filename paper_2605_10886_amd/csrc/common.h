// Shared host/device helpers of the HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/loka.h"

#define LOKA_HIP_TRY(expr)                        \
    do {                                          \
        hipError_t e__ = (expr);                  \
        if (e__ != hipSuccess) return LOKA_ERR_HIP; \
    } while (0)

namespace loka {

constexpr float kE4M3Max = 448.0f;
constexpr float kAmaxFloor = 1e-12f;

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// scale modes 3..6 are the block recipes (1 x 128 activations, 128 x 128 weights); 5 and 6 have power-of-two scales
static inline bool scale_mode_is_block(int m) { return m >= LOKA_SCALE_BLOCK_1x128 && m <= LOKA_SCALE_BLOCK_128x128_POW2; }
static inline bool scale_mode_is_pow2(int m) { return m == LOKA_SCALE_BLOCK_1x128_POW2 || m == LOKA_SCALE_BLOCK_128x128_POW2; }

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }
// low / high bf16 of a 32-bit word holding two consecutive elements
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Round-to-nearest-even narrowing of a finite fp32 to bf16 bits.
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7F800000u) == 0x7F800000u) return (u >> 16) | ((u & 0x007FFFFFu) ? 0x40u : 0u);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
// Two fp32 -> packed bf16 (round-to-nearest-even) with the gfx950 convert instruction.
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const bf16x2_t v = __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t);
    return __builtin_bit_cast(uint32_t, v);
}

// OCP e4m3 cast of four fp32 values (round-to-nearest-even by the gfx950 convert
// instruction, which encodes OCP e4m3 on this target).  The clamp comes first: the
// hardware maps magnitudes of 480 and above to NaN instead of saturating.
__device__ __forceinline__ float clamp448(float t) { return __builtin_fminf(__builtin_fmaxf(t, -kE4M3Max), kE4M3Max); }
__device__ __forceinline__ uint32_t e4m3x4(float t0, float t1, float t2, float t3) {
    int pk = 0;
    pk = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(t0), clamp448(t1), pk, false);
    pk = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(t2), clamp448(t3), pk, true);
    return static_cast<uint32_t>(pk);
}

// amax floor, dequantization scale and quantization factor of one scale group:
// each a single IEEE fp32 division.
__device__ __forceinline__ void group_scale(float amax, float& scale, float& inv) {
    float a = amax < kAmaxFloor ? kAmaxFloor : amax;
    scale = a / kE4M3Max;
    inv = kE4M3Max / a;
}

// Power-of-two block modes: the smallest power of two s with amax / s <= 448, from the bits of amax
// (448 = 1.75 * 2^8: amax = 1.f * 2^e needs s = 2^(e - 8) when 1.f <= 1.75, else 2^(e - 7)); inv = 1 / s, exact.
__device__ __forceinline__ void group_scale_pow2(float amax, float& scale, float& inv) {
    const float a = amax < kAmaxFloor ? kAmaxFloor : amax;
    const uint32_t b = __float_as_uint(a);
    const uint32_t e = (b >> 23) - 8u + ((b & 0x7FFFFFu) > 0x600000u ? 1u : 0u);      // biased exponent of s
    scale = __uint_as_float(e << 23);
    inv = __uint_as_float((254u - e) << 23);
}
__device__ __forceinline__ void group_scale_any(bool pow2, float amax, float& scale, float& inv) {
    if (pow2) group_scale_pow2(amax, scale, inv);
    else group_scale(amax, scale, inv);
}

__device__ __forceinline__ float wave_shfl_xor(float v, int mask) { return __shfl_xor(v, mask, 64); }

}  // namespace loka
