// Shared device/host helpers for the gfx950 BiGLA + locality-gate kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vig {

// ---- bf16 storage <-> fp32 ------------------------------------------------------------------
// bf16 is the upper half of an IEEE fp32.  Widening is a shift; narrowing rounds to nearest even.
struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float bf16_lo_to_f32(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // NaN stays NaN (quiet)
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// Two fp32 -> one dword of bf16, round to nearest even, in one instruction (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t a = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2_t));
}

template <typename T>
struct io;  // element load/store in fp32 terms

template <>
struct io<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};

template <>
struct io<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t *p) { return __uint_as_float(uint32_t(p->bits) << 16); }
    static __device__ __forceinline__ void store(bf16_t *p, float v) { p->bits = uint16_t(f32_to_bf16_bits(v)); }
};

}  // namespace vig
