// Helpers of the kernels that run fp32 products on the bf16 matrix instruction: an fp32 value is
// cut (by truncation, remainders computed exactly) into three bf16 pieces that add up to it, and
// of the nine piece products of a * b the six of weight >= 2^-16 are accumulated in fp32.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace ag {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));     // 16 bytes of packed bf16 pieces

// v_mfma_f32_32x32x16_bf16: lane l holds A[l & 31][8 (l >> 5) + 0..7] and B[8 (l >> 5) + 0..7][l & 31]
// (element t of the eight in the low / high half of word t / 2); result register r holds
// D[8 (r / 4) + 4 (l >> 5) + (r & 3)][l & 31].
__device__ __forceinline__ floatx16 mfma16(const u32x4 &a, const u32x4 &b, const floatx16 &c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// p[0] + p[1] + p[2] == h exactly (each piece an fp32 number whose low 16 bits are zero)
__device__ __forceinline__ void cut3(float h, uint32_t (&p)[3])
{
    p[0] = __float_as_uint(h) & 0xffff0000u;
    const float r1 = h - __uint_as_float(p[0]);
    p[1] = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(p[1]);
    p[2] = __float_as_uint(r2) & 0xffff0000u;
}

// Eight fp32 values -> three operands of eight bf16 pieces each (value t in slot t).
__device__ __forceinline__ void cut3x8(const float (&v)[8], u32x4 (&out)[3])
{
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        uint32_t lo[3], hi[3];
        cut3(v[2 * w], lo);
        cut3(v[2 * w + 1], hi);
#pragma unroll
        for (int s = 0; s < 3; ++s) out[s][w] = (lo[s] >> 16) | hi[s];
    }
}

// acc += a * b for operands cut into pieces: the six products of weight >= 2^-16, smallest first
__device__ __forceinline__ floatx16 mfma16_b3(const u32x4 (&a)[3], const u32x4 (&b)[3], floatx16 c)
{
    c = mfma16(a[2], b[0], c);
    c = mfma16(a[0], b[2], c);
    c = mfma16(a[1], b[1], c);
    c = mfma16(a[1], b[0], c);
    c = mfma16(a[0], b[1], c);
    c = mfma16(a[0], b[0], c);
    return c;
}

}  // namespace ag
