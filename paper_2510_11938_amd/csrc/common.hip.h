// Shared device helpers for the gfx950 kernels: bf16 encode/decode, wavefront
// (64-lane) reductions, 16-byte vector access.  Device code only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fxp {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kBlockTokens = 16;   // tokens per KV cache block (fixed by the ABI)

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;   // one MFMA operand
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;      // 16x16 MFMA accumulator

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16-byte memory vector
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// float -> bf16, round to nearest even; NaN stays NaN.  One v_cvt_pk_bf16_f32 per pair
// (gfx950 converts in hardware; it agrees with add-0x7fff-plus-lsb rounding on every one of
// the 2^32 float patterns that is not a NaN).
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return (uint16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

__device__ __forceinline__ u32x4 ld16(const void *p) { return *reinterpret_cast<const u32x4 *>(p); }
__device__ __forceinline__ void st16(void *p, u32x4 v) { *reinterpret_cast<u32x4 *>(p) = v; }

// Sum / max over the 64 lanes of a wavefront; every lane gets the result.
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

}  // namespace fxp
