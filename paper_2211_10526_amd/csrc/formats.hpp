// Vector types, lane-crossing helpers and the two 16-bit I/O formats of the matrix-core kernels
// (gfx950, wave64).
#pragma once

#include "common.hpp"

namespace castling {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;

// x + (value of x in another lane chosen by a DPP control)
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false);
    return x + __int_as_float(y);
}

constexpr int kDppQuadXor1 = 0xB1;       // quad_perm [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;       // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141; // lane i <-> 7-i inside each group of 8
constexpr int kDppRowRor8 = 0x128;       // rotate by 8 inside each row of 16

// Sum over LANES consecutive lanes (4, 8 or 16); every lane of the group gets the sum.
template <int LANES>
__device__ __forceinline__ float row_group_sum(float x)
{
    x = dpp_add<kDppQuadXor1>(x);
    x = dpp_add<kDppQuadXor2>(x);
    if constexpr (LANES >= 8) x = dpp_add<kDppRowHalfMirror>(x);
    if constexpr (LANES >= 16) x = dpp_add<kDppRowRor8>(x);
    return x;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    bf16x2_t r;
    r[0] = static_cast<__bf16>(lo);
    r[1] = static_cast<__bf16>(hi);
    return __builtin_bit_cast(uint32_t, r);
}

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;

// The two 16-bit I/O formats of the matrix-core kernels.  Values travel as raw bits (u32x4_t =
// 8 values, s16x4_t = 4 values, uint32_t = 2 values) and are typed only where they are converted
// or multiplied.  The operand tables hold S * table_scale and ksum * table_scale; the apply
// side multiplies its products by table_unscale.  fp16 tables are scaled by 1 / N: |S_ij| and
// |ksum_i| are at most N max|v| resp. N, so the scaled entries cannot overflow fp16 unless the
// inputs themselves are at its limit.
struct Bf16Fmt {
    static constexpr bool kHalf = false;
    static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
    static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
    static __device__ __forceinline__ float one(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }
    static __device__ __forceinline__ uint32_t pack(float a, float b) { return pack_bf16x2(a, b); }
    static __host__ __device__ __forceinline__ float table_scale(int) { return kInvPi; }
    static __host__ __device__ __forceinline__ float table_unscale(int) { return 1.0f; }
    static __device__ __forceinline__ f32x16_t mfma32(u32x4_t a, u32x4_t b, f32x16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4_t mfma16(u32x4_t a, u32x4_t b, f32x4_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4_t mfma4(s16x4_t a, s16x4_t b, f32x4_t c)
    {
        return __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, b, c, 0, 0, 0);
    }
    static constexpr uint32_t kOneLo = 0x00003f80u, kOneHi = 0x3f800000u;  // (1, 0) and (0, 1)
    // a.lo * b.lo + a.hi * b.hi + c in fp32 (v_dot2c_f32_bf16)
    static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
    {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                               __builtin_bit_cast(bf16x2_t, b), c, false);
    }
};

struct F16Fmt {
    static constexpr bool kHalf = true;
    static __device__ __forceinline__ float one(uint16_t b) { return static_cast<float>(__builtin_bit_cast(_Float16, b)); }
    static __device__ __forceinline__ float lo(uint32_t w) { return one(static_cast<uint16_t>(w)); }
    static __device__ __forceinline__ float hi(uint32_t w) { return one(static_cast<uint16_t>(w >> 16)); }
    // round to nearest even; beyond the fp16 range the result is infinity
    static __device__ __forceinline__ uint32_t pack(float a, float b)
    {
        f16x2_t r;
        r[0] = static_cast<_Float16>(a);
        r[1] = static_cast<_Float16>(b);
        return __builtin_bit_cast(uint32_t, r);
    }
    static __host__ __device__ __forceinline__ float table_scale(int N) { return kInvPi / static_cast<float>(N); }
    static __host__ __device__ __forceinline__ float table_unscale(int N) { return static_cast<float>(N); }
    static __device__ __forceinline__ f32x16_t mfma32(u32x4_t a, u32x4_t b, f32x16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4_t mfma16(u32x4_t a, u32x4_t b, f32x4_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4_t mfma4(s16x4_t a, s16x4_t b, f32x4_t c)
    {
        return __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(f16x4_t, a),
                                                  __builtin_bit_cast(f16x4_t, b), c, 0, 0, 0);
    }
    static constexpr uint32_t kOneLo = 0x00003c00u, kOneHi = 0x3c000000u;  // (1, 0) and (0, 1)
    // a.lo * b.lo + a.hi * b.hi + c in fp32 (v_dot2c_f32_f16)
    static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
    {
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, a), __builtin_bit_cast(f16x2_t, b),
                                      c, false);
    }
};

}  // namespace castling
