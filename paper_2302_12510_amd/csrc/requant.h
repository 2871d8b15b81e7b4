// Write-back encoder for the matrix-product epilogue (Sec. III-B: results leave the array as DyBit
// codes): one fp32 value -> the DyBit code nearest to value / scale in exact arithmetic, ties to the
// even magnitude code -- the same function the stand-alone quantize pass computes, with the format
// as run-time (wave-uniform) parameters so that one epilogue serves every output format.
//
// Fast path: q = min(|x| * fl(1/s), vmax) is within 2^-23 (relative) of the true quotient t.  The real-valued
// code c(t) -- t * 2^(m-1) below 1, then the inverse of the decoder's bit-pattern identity -- is
// piecewise linear and continuous, and the decision points between codes are its half-integers.  One
// expression yields n = 2^m - c(q) over the whole range: with q' = q * 2^-126 (a subnormal float below 1,
// whose bits are linear in q), n = bitcast(((127 + m) << 23) - bits(q')).  n is rounded to G fractional
// bits by one magic-number addition; unless those bits read exactly one half, q and t lie on the same
// side of every decision point.  When they do read one half (one element in 2^G) the nearest decision
// point is the midpoint above code floor(c), and the sign of fma(-s, midpoint, |x|), which is exact,
// settles the side; zero is a tie and goes to the even code.  A NaN becomes q = 0, hence code 0
// (v_med3_f32 returns the minimum of its other operands for a NaN).
#ifndef DYBIT_REQUANT_H
#define DYBIT_REQUANT_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dybit {

// G: fractional bits kept by the magic-number rounding.  The error of c is below 1.5 * 2^(m-24), so
// G = 13 serves every format (m <= 8), and 2^m + magic stays inside the magic number's binade.
// The magic number carries one half more than 1.5 * 2^(23-G): the rounded sum is the same number of units of
// 2^-G plus that half (adding an even number of units changes neither the rounding nor its tie rule), so a
// fraction of exactly one half reads as G zero bits and is found by one shift.
struct Requant {
    static constexpr int G = 13;
    static constexpr uint32_t kMagic = (((uint32_t)(127 + 23 - G) << 23) | 0x400000u) + (1u << (G - 1));   // 1.5 * 2^(23-G) + 1/2
    static constexpr uint32_t kRound = kMagic + (1u << (G - 1));
    static constexpr uint32_t kFracMask = (1u << G) - 1u;
    float rinv;         // fl(1 / s)
    float p, s2;        // power of two that brings s into [1, 2), and s * p
    float vmax;         // 2^(m-1): the largest magnitude
    float inv_grid;     // 2^-(m-1)
    float two_m;        // 2^m
    float floor_x;      // lower clamp of the input when a decision is settled: -inf (signed: |x| follows) or 0 (unsigned)
    uint32_t abs_mask;  // clears the sign of x / s for a signed format, keeps it for an unsigned one (negative -> 0)
    uint32_t recip_k;   // (254 + m - 1) << 23: constant of the bit-pattern subtraction
    uint32_t recip_sub; // (127 + m) << 23: the same for an argument scaled by 2^-126
    uint32_t m;         // magnitude bits
    uint32_t half;      // 2^(m-1): first code of the part above 1
    uint32_t sign_mask, sign_shift;
    bool is_signed;
    bool ok;            // scale is positive, finite and within [2^-100, 2^100]
};

__device__ __forceinline__ Requant make_requant(const float *scale, int bits, int is_signed)
{
    Requant r;
    const float s = *scale;
    const uint32_t e = (__float_as_uint(s) >> 23) & 0xffu;
    r.ok = s > 0.0f && e >= 27u && e <= 227u;
    r.rinv = 1.0f / s;
    r.p = __uint_as_float((254u - e) << 23);
    r.s2 = s * r.p;
    const int m = is_signed ? bits - 1 : bits;
    r.m = (uint32_t)m;
    r.vmax = (float)(1u << (m - 1));
    r.inv_grid = __uint_as_float((uint32_t)(127 - (m - 1)) << 23);
    r.two_m = (float)(1u << m);
    r.floor_x = is_signed ? -__builtin_inff() : 0.0f;
    r.abs_mask = is_signed ? 0x7fffffffu : 0xffffffffu;
    r.recip_k = (uint32_t)(254 + m - 1) << 23;
    r.recip_sub = (uint32_t)(127 + m) << 23;
    r.half = 1u << (m - 1);
    r.is_signed = is_signed != 0;
    r.sign_mask = is_signed ? (1u << m) : 0u;
    r.sign_shift = (uint32_t)(31 - m);
    return r;
}

// Fast path, first half: the bit pattern of (2^m - c) + magic for the value x.  The G low bits are the
// rounded fraction of c plus one half; requant_needs_settling() says whether the fraction is one half.  A NaN gives c = 0.
__device__ __forceinline__ uint32_t requant_rounded(float x, const Requant &r)
{
    const float t = __uint_as_float(__float_as_uint(x * r.rinv) & r.abs_mask);  // |x| / s, or x / s (negative: clamped to 0 below)
    const float q = __builtin_amdgcn_fmed3f(t, 0.0f, r.vmax);                   // saturated; NaN -> 0
    const float qs = q * __uint_as_float(1u << 23);                             // q * 2^-126
    const float n = __uint_as_float(r.recip_sub - __float_as_uint(qs));         // 2^m - c (-2^m should the median of -0, 0, vmax be -0)
    return __float_as_uint(fabsf(n) + __uint_as_float(Requant::kMagic));
}

__device__ __forceinline__ bool requant_needs_settling(uint32_t zb)
{
    return (zb & Requant::kFracMask) == 0u;
}

// The same test in a form that accumulates with an unsigned minimum: zero exactly when the fraction is
// one half (the G low bits, moved to the top of the word, are all zero).
__device__ __forceinline__ uint32_t requant_settle_key(uint32_t zb)
{
    return zb << (32 - Requant::G);
}

// Fast path, second half: the magnitude code, c rounded half up (the low m bits of the difference:
// the 2^m of the upper form drops out).
__device__ __forceinline__ uint32_t requant_magnitude(uint32_t zb, const Requant &r)
{
    return __builtin_amdgcn_ubfe(Requant::kRound - zb, Requant::G, r.m);
}

// Exact decision at the midpoint between magnitude codes `code - 1` and `code`, for a value whose
// rounded fraction read one half (so code >= 1; a NaN never gets here, its fraction reads zero).
__device__ __forceinline__ uint32_t requant_settle(float x, uint32_t code, const Requant &r)
{
    const float ax = fabsf(fmaxf(x, r.floor_x));
    const uint32_t lo = code - 1u;
    const float h = (float)lo + 0.5f;
    const float mid = lo < r.half ? h * r.inv_grid : __uint_as_float(r.recip_k - __float_as_uint(r.two_m - h));
    const float d = fmaf(-r.s2, mid, ax * r.p);                     // sign(|x| - s * mid), exact
    return (d > 0.0f || (d == 0.0f && (lo & 1u))) ? code : lo;
}

// Sign bit for a signed format (sign_mask is 0 for an unsigned one); a zero magnitude never carries it.
__device__ __forceinline__ uint32_t requant_with_sign(uint32_t mag, float x, const Requant &r)
{
    const uint32_t sign = (__float_as_uint(x) >> r.sign_shift) & r.sign_mask;
    return mag ? (mag | sign) : 0u;
}

// One value, all steps (the epilogue below runs the steps in phases over 16 values instead).
__device__ __forceinline__ uint32_t requant_code(float x, const Requant &r)
{
    const uint32_t zb = requant_rounded(x, r);
    uint32_t mag = requant_magnitude(zb, r);
    if (requant_needs_settling(zb)) mag = requant_settle(x, mag, r);
    return requant_with_sign(mag, x, r);
}

// ---- packing across lanes -----------------------------------------------------------------------
// In the matrix-core result layout the 32 lanes of a half-wave hold 32 consecutive columns of one
// row, so the codes of neighbouring lanes are neighbours in the packed row.  8-bit codes need no
// packing: every lane stores its byte (32 consecutive bytes per row and instruction, the same
// footprint as eight lanes storing words).  4-bit codes: a lane pair ORs its two nibbles together
// with one data-parallel lane permute and the even lane stores the byte.  6-bit codes: each lane
// shifts its code to its position inside a 32-bit word, the four lanes that share 24 bits OR their
// parts together (two permutes), a third permute fetches the next group's 24 bits (lanes 12 .. 15 of a row of 16
// read zero there and store nothing), and 16 lanes' 96 bits leave as three words.  No LDS, no memory;
// all 64 lanes must be active.
__device__ __forceinline__ uint32_t or_quad(uint32_t w)
{
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0xB1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x4E, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
    return w;
}

// Where a lane's word goes inside the packed row and whether the lane is the one that stores it.
// col = column of the lane's value (a multiple of 32 plus lane % 32).
struct PackSlot {
    uint32_t shift;      // position of the lane's code inside the group's byte or word(s)
    uint32_t byte_off;   // byte offset of the lane's byte (4-, 8-bit) or word (6-bit) inside the packed row
    bool stores;
};

template <int BITS>
__device__ __forceinline__ PackSlot pack_slot(int lane, uint32_t col)
{
    PackSlot p;
    if (BITS == 8) {
        p.shift = 0;               p.byte_off = col;            p.stores = true;
    } else if (BITS == 4) {
        p.shift = (lane & 1) * 4;  p.byte_off = col >> 1;       p.stores = (lane & 1) == 0;
    } else {                                                    // 6-bit: 16 codes = three words
        const uint32_t k = (lane >> 2) & 3;                     // which group of four inside the 16
        p.shift = (lane & 3) * 6;  p.byte_off = (col >> 4) * 12 + 4 * k;   p.stores = (lane & 3) == 0 && k < 3;
    }
    return p;
}

template <int BITS>
__device__ __forceinline__ uint32_t pack_word(uint32_t code, int lane, const PackSlot &p)
{
    if (BITS == 8) return code;
    if (BITS == 4) {
        const uint32_t w = code << p.shift;
        return w | (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0xB1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]: the neighbour's nibble
    }
    uint32_t w = or_quad(code << p.shift);
    if (BITS == 6) {
        // four lanes hold 24 bits; word k of the three takes the rest from the next group of four
        const uint32_t k = (lane >> 2) & 3;
        const uint32_t next = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x104, 0xf, 0xf, true);   // row_shl:4: lane i reads lane i + 4 of its row of 16
        w = (w >> (8 * k)) | (next << (24 - 8 * k));
    }
    return w;
}

}  // namespace dybit
#endif
