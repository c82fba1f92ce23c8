// Three-piece bf16 operands for the bf16 matrix pipeline.
//
// x = h + m + l with h = bf16(x), m = bf16(x - h), l = bf16(x - h - m) (round to nearest even; both
// differences are exact in fp32), so the three pieces carry 24 significant bits.  A product of two such
// numbers is taken as the six piece products that matter,
//     x*y ~ h*h' + (h*m' + m*h') + m*m' + (h*l' + l*h'),
// the dropped ones (m*l', l*m', l*l') being below 2^-24 relative.  Each piece product is exact in fp32 and
// the products are summed in fp32 by v_mfma_f32_16x16x32_bf16, so the result has the accuracy of an fp32
// dot product while running on the bf16 matrix pipeline and, unlike the fp32 matrix instructions,
// concurrently with the vector ALU.  Used by the stage convolution (conv_split.hip) and by the patch Gram.
#pragma once

#include "ddcca_internal.h"

namespace ddcca {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// One operand of v_mfma_f32_16x16x32_bf16: 8 bf16 values = four 32-bit words of packed pairs.
union SplitOperand {
    bf16x8 v;
    unsigned int w[4];
};

__device__ __forceinline__ unsigned bf16_bits(__bf16 b) { return (unsigned)__builtin_bit_cast(unsigned short, b); }

// The three bf16 pieces of x, as 16-bit patterns.
__device__ __forceinline__ void split3(float x, unsigned &h, unsigned &m, unsigned &l)
{
    const __bf16 bh = (__bf16)x;
    const float r1 = x - (float)bh;
    const __bf16 bm = (__bf16)r1;
    const float r2 = r1 - (float)bm;
    const __bf16 bl = (__bf16)r2;
    h = bf16_bits(bh);
    m = bf16_bits(bm);
    l = bf16_bits(bl);
}

typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// bf16(a) | bf16(b) << 16, both rounded to nearest even (one packed conversion).
__device__ __forceinline__ unsigned bf16_pair(float a, float b)
{
    return __builtin_bit_cast(unsigned, __builtin_convertvector(floatx2{a, b}, bf16x2));
}

// The three pieces of the pair (a, b), each as a packed word bf16(a) | bf16(b) << 16.
__device__ __forceinline__ void split3_pair(float a, float b, unsigned &h, unsigned &m, unsigned &l)
{
    h = bf16_pair(a, b);
    const float ra = a - __uint_as_float(h << 16), rb = b - __uint_as_float(h & 0xffff0000u);
    m = bf16_pair(ra, rb);
    l = bf16_pair(ra - __uint_as_float(m << 16), rb - __uint_as_float(m & 0xffff0000u));
}

}  // namespace ddcca
