// Device-side helpers shared by the DyBit kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dybit.h"

namespace dybit {

__host__ __device__ inline int mag_bits(int bits, int is_signed) { return is_signed ? bits - 1 : bits; }

// Magnitude code -> value (Eq. 1 / Table I) without a table.
//
// Codes whose first bit is 0 are the fraction c / 2^(m-1).  For the others let
// n = 2^m - c (1 <= n <= 2^(m-1)).  A code with i leading ones, a zero and the
// k-bit fraction x has n = 2^(k+1) - x, so float(n) has exponent k (k+1 when
// x == 0) and mantissa 1 - x/2^k.  Subtracting its bit pattern from the constant
// (bias + bias + m-1) << 23 turns exponent k = m-i-1 into i-1 and the mantissa
// into x/2^k, i.e. exactly 2^(i-1) (1 + x/2^k); the borrow of the integer
// subtraction handles x == 0 and the all-ones code (n = 1 -> 2^(m-1)).
__device__ __forceinline__ float magnitude_value(uint32_t c, int m)
{
    if ((c >> (m - 1)) == 0) return (float)c * __uint_as_float((uint32_t)(127 - (m - 1)) << 23);
    const float n = (float)((1u << m) - c);
    return __uint_as_float(((uint32_t)(254 + m - 1) << 23) - __float_as_uint(n));
}

// Full code (sign-magnitude) -> value; sign=1, magnitude=0 is +0.
__device__ __forceinline__ float code_value(uint32_t code, int bits, int is_signed)
{
    const int m = mag_bits(bits, is_signed);
    const uint32_t c = code & ((1u << m) - 1);
    const float v = magnitude_value(c, m);
    return (is_signed && (code >> m) && c) ? -v : v;
}

}  // namespace dybit
