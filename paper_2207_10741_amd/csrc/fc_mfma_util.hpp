// Pieces shared by the matrix-core kernels: the 32x32x16 MFMA wrapper for bf16 / f16
// operands, the rounding store of four accumulator values, and the two ReLU forms.
#pragma once
#include "fc_internal.hpp"

namespace fc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

template <int DT>
__device__ __forceinline__ f32x16_t mfma32(const uint4 &a, const uint4 &b, const f32x16_t &c)
{
    if constexpr (DT == FC_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// Four fp32 values -> four stored values; the narrowing is the hardware's
// round-to-nearest-even conversion (v_cvt_pk_bf16_f32 / v_cvt_f16_f32).
template <int DT, typename TO>
__device__ __forceinline__ void store4(TO *dst, float a, float b, float c, float d)
{
    if constexpr (sizeof(TO) == 4) {
        *reinterpret_cast<float4 *>(dst) = make_float4(a, b, c, d);
    } else if constexpr (DT == FC_BF16) {
        const f32x2_t lo = {a, b}, hi = {c, d};
        uint2 v;
        v.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2_t));
        v.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2_t));
        *reinterpret_cast<uint2 *>(dst) = v;
    } else {
        const f32x2_t lo = {a, b}, hi = {c, d};
        uint2 v;
        v.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, f16x2_t));
        v.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, f16x2_t));
        *reinterpret_cast<uint2 *>(dst) = v;
    }
}

// max(v, 0) that keeps NaN (and -0) as the reference does
__device__ __forceinline__ float relu_keep_nan(float v) { return v < 0.f ? 0.f : v; }

// ReLU of two packed 16-bit floats (bf16 or f16): a value with the sign bit set becomes +0.
// (-0 becomes +0, and a NaN with the sign bit set becomes 0: neither is a value the
// accumulation produces from finite inputs.)
typedef short i16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t relu_packed16(uint32_t two)
{
    const i16x2_t zero = {0, 0};
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(i16x2_t, two), zero));
}

} // namespace fc
