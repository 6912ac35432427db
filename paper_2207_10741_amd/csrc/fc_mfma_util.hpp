// Pieces shared by the matrix-core kernels: the MFMA wrapper (32x32x16 for bf16 / f16
// operands, 32x32x64 for fp8), the rounding store of four accumulator values, and the two ReLU forms.
#pragma once
#include "fc_internal.hpp"

namespace fc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

typedef int i32x8_t __attribute__((ext_vector_type(8)));

// Bytes of a 128-byte LDS row that one matrix instruction consumes: 32 for the 16-bit types
// (v_mfma_f32_32x32x16: a lane holds 8 elements = one 16-byte piece of its row), 64 for fp8
// (v_mfma_f32_32x32x64_f8f6f4: a lane holds 32 elements = two adjacent pieces).
template <int DT> constexpr uint32_t kStepBytes = DT == FC_FP8 ? 64u : 32u;

// One lane's share of a matrix operand.  The 16-byte piece index of a lane in step kk is
// 2*kk + (lane >> 5) for the 16-bit types and 4*kk + 2*(lane >> 5) + {0, 1} for fp8; the
// caller passes the byte address of the first piece (swizzle applied) and the second one is
// the same address with bit 4 flipped (the swizzle is an XOR, so it commutes).
template <int DT> struct Frag {
    uint4 v;
    __device__ __forceinline__ void load(const unsigned char *base, uint32_t off)
    {
        v = *reinterpret_cast<const uint4 *>(base + off);
    }
};
template <> struct Frag<FC_FP8> {
    uint4 v, v2;
    __device__ __forceinline__ void load(const unsigned char *base, uint32_t off)
    {
        v = *reinterpret_cast<const uint4 *>(base + off);
        v2 = *reinterpret_cast<const uint4 *>(base + (off ^ 16u));
    }
};

// acc += a * b over one step of the reduction.  Both operands hold the same reduction
// elements in the same registers, so the product does not depend on how the hardware numbers
// them.  fp8 is the E4M3 format (format selectors 0), operands unscaled.
template <int DT>
__device__ __forceinline__ f32x16_t mfma32(const Frag<DT> &a, const Frag<DT> &b, const f32x16_t &c)
{
    if constexpr (DT == FC_BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a.v),
                                                       __builtin_bit_cast(bf16x8_t, b.v), c, 0, 0, 0);
    } else if constexpr (DT == FC_F16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a.v),
                                                      __builtin_bit_cast(f16x8_t, b.v), c, 0, 0, 0);
    } else {
        const i32x8_t av = {(int)a.v.x, (int)a.v.y, (int)a.v.z, (int)a.v.w,
                            (int)a.v2.x, (int)a.v2.y, (int)a.v2.z, (int)a.v2.w};
        const i32x8_t bv = {(int)b.v.x, (int)b.v.y, (int)b.v.z, (int)b.v.w,
                            (int)b.v2.x, (int)b.v2.y, (int)b.v2.z, (int)b.v2.w};
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, c, 0, 0, 0, 0, 0, 0);
    }
}

// the same for operands already held as one 16-byte piece per lane (16-bit types only)
template <int DT>
__device__ __forceinline__ f32x16_t mfma32(const uint4 &a, const uint4 &b, const f32x16_t &c)
{
    static_assert(DT != FC_FP8, "fp8 operands are two pieces per lane");
    Frag<DT> fa, fb;
    fa.v = a;
    fb.v = b;
    return mfma32<DT>(fa, fb, c);
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// Four fp32 values -> four stored values; the narrowing is the hardware's
// round-to-nearest-even conversion (v_cvt_pk_bf16_f32 / v_cvt_f16_f32).
// a value held to the E4M3 range; NaN stays NaN
__device__ __forceinline__ float sat_e4m3(float v)
{
    return v != v ? v : __builtin_amdgcn_fmed3f(v, -448.f, 448.f);
}

template <int DT, typename TO>
__device__ __forceinline__ void store4(TO *dst, float a, float b, float c, float d)
{
    if constexpr (sizeof(TO) == 4) {
        *reinterpret_cast<float4 *>(dst) = make_float4(a, b, c, d);
    } else if constexpr (sizeof(TO) == 1) {
        // v_cvt_pk_fp8_f32 rounds two values to nearest even (E4M3 on gfx950); magnitudes are
        // held at 448 first so that the result does not depend on its overflow behaviour
        a = sat_e4m3(a); b = sat_e4m3(b); c = sat_e4m3(c); d = sat_e4m3(d);
        int r = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
        r = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, r, true);
        *reinterpret_cast<uint32_t *>(dst) = (uint32_t)r;
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

// ReLU of four packed 8-bit floats: a code with the sign bit set becomes +0.
__device__ __forceinline__ uint32_t relu_packed8(uint32_t four)
{
    return four & ~(((four >> 7) & 0x01010101u) * 0xFFu);
}

} // namespace fc
