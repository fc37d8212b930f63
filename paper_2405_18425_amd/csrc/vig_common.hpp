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

// ---- vector types, packing and matrix-core helpers shared by the MFMA kernels ---------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

// 2^x on the hardware's own instruction (v_exp_f32): no range handling, an underflow to 0 is the
// right limit wherever it is used
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack2(float lo, float hi) { return pack_bf16x2(lo, hi); }
__device__ __forceinline__ uint2 pack4(const f32x4 &p) { return make_uint2(pack2(p[0], p[1]), pack2(p[2], p[3])); }
__device__ __forceinline__ f32x4 unpack4(const uint2 &u)
{
    return f32x4{bf16_lo_to_f32(u.x), bf16_hi_to_f32(u.x), bf16_lo_to_f32(u.y), bf16_hi_to_f32(u.y)};
}

__device__ __forceinline__ f32x4 mfma(bf16x8 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// lanes whose DPP source falls outside the 16-lane row receive 0
template <int CTRL>
__device__ __forceinline__ float dpp_or_zero(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}

// Inclusive scan over the 16 lanes of a DPP row: prefix sums (SUFFIX 0) or suffix sums (SUFFIX 1).
template <int SUFFIX>
__device__ __forceinline__ float row_scan(float x)
{
    if (SUFFIX == 0) {
        x += dpp_or_zero<0x111>(x);  // row_shr:1
        x += dpp_or_zero<0x112>(x);
        x += dpp_or_zero<0x114>(x);
        x += dpp_or_zero<0x118>(x);
    } else {
        x += dpp_or_zero<0x101>(x);  // row_shl:1
        x += dpp_or_zero<0x102>(x);
        x += dpp_or_zero<0x104>(x);
        x += dpp_or_zero<0x108>(x);
    }
    return x;
}

// Transposing LDS read: the 16 lanes of a row fetch a 4 (rows) x 16 (columns) bf16 patch of a
// row-major tile; lane n of the row receives the 4 rows of column n and supplies the address of
// row n/4, columns 4*(n%4).. of the patch.
__device__ __forceinline__ s16x4 lds_read_tr(const uint16_t *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(p));
}

__device__ __forceinline__ bf16x8 join(s16x4 lo, s16x4 hi)
{
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// Buffer resource over `extent_bytes` bytes at p.  Offsets into it are 32 bits wide, and an access
// beyond the extent returns zeros (load) or is dropped (store): the bounds check of the hardware
// stands in for clamps, branches and selects on ragged ends.  The resource is the same in every
// lane; saying so keeps it in scalar registers.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t slab_resource(const void *p, unsigned extent_bytes)
{
    const uintptr_t a = reinterpret_cast<uintptr_t>(p);
    // (readfirstlane returns a signed int: widen through unsigned, not by sign extension)
    const uintptr_t lo = unsigned(__builtin_amdgcn_readfirstlane(int(unsigned(a))));
    const uintptr_t hi = unsigned(__builtin_amdgcn_readfirstlane(int(unsigned(a >> 32))));
    const unsigned kRawDwords = 0x00020000u;  // untyped 32-bit data, bounds check on the byte offset
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(lo | (hi << 32)), 0,
                                             int(unsigned(__builtin_amdgcn_readfirstlane(int(extent_bytes)))),
                                             int(kRawDwords));
}

// log(sigmoid(z)) = min(z, 0) - log(1 + exp(-|z|)), finite for every finite z.  The bare hardware
// exp2 / log2 serve: the exponential's argument is <= 0 (an underflow to 0 is the right limit) and
// the logarithm's lies in [1, 2], so neither needs the range handling of the library functions,
// which costs more vector instructions than the two transcendentals themselves.
__device__ __forceinline__ float log_sigmoid(float z)
{
    const float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
    const float e = __builtin_amdgcn_exp2f(-kLog2e * fabsf(z));
    return fmaf(-kLn2, __builtin_amdgcn_logf(1.f + e), fminf(z, 0.f));
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
