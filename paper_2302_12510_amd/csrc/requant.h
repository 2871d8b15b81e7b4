// Write-back encoder for the matrix-product epilogue (Sec. III-B: results leave the array as DyBit
// codes): one fp32 value -> the DyBit code nearest to value / scale in exact arithmetic, ties to the
// even magnitude code -- the same function the stand-alone quantize pass computes, with the format
// as run-time (wave-uniform) parameters so that one epilogue serves every output format.
//
// Fast path: q = |x| * fl(1/s) is within 2^-23 (relative) of the true quotient t.  The real-valued
// code c(t) -- t * 2^(m-1) below 1, and 2^m minus the value whose bit pattern is a constant minus
// t's above -- is piecewise linear and continuous, and the decision points between codes are its
// half-integers.  c is rounded to G fractional bits by one magic-number addition; unless those
// bits read exactly one half, q and t lie on the same side of every decision point.  When they do
// read one half (one element in 2^G) the nearest decision point is the midpoint above code
// floor(c), and the sign of fma(-s, midpoint, |x|), which is exact, settles the side; zero is a
// tie and goes to the even code.
#ifndef DYBIT_REQUANT_H
#define DYBIT_REQUANT_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dybit {

struct Requant {
    static constexpr int G = 12;                                                       // 2^(m-23) << 2^-(G+1) for m <= 8
    static constexpr uint32_t kMagic = ((uint32_t)(127 + 23 - G) << 23) | 0x400000u;   // 1.5 * 2^(23-G)
    static constexpr uint32_t kRound = kMagic + (1u << (G - 1));
    float rinv;         // fl(1 / s)
    float p, s2;        // power of two that brings s into [1, 2), and s * p
    float vmax;         // 2^(m-1): the largest magnitude
    float neg_grid;     // -2^(m-1): -(codes per unit) on the fraction grid below 1
    float inv_grid;     // 2^-(m-1)
    float two_m;        // 2^m
    uint32_t recip_k;   // (254 + m - 1) << 23: constant of the bit-pattern subtraction
    uint32_t top;       // 2^m - 1, the all-ones magnitude
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
    r.vmax = (float)(1u << (m - 1));
    r.neg_grid = -r.vmax;
    r.inv_grid = __uint_as_float((uint32_t)(127 - (m - 1)) << 23);
    r.two_m = (float)(1u << m);
    r.recip_k = (uint32_t)(254 + m - 1) << 23;
    r.top = (1u << m) - 1u;
    r.half = 1u << (m - 1);
    r.is_signed = is_signed != 0;
    r.sign_mask = is_signed ? (1u << m) : 0u;
    r.sign_shift = (uint32_t)(31 - m);
    return r;
}

// Exact decision at the midpoint between magnitude codes `code - 1` and `code`.  ax = |x| (signed
// formats) or max(x, 0); NaN -> 0.
__device__ __forceinline__ uint32_t requant_settle(float x, float ax, uint32_t code, const Requant &r)
{
    if (x != x) return 0u;
    const uint32_t lo = code - 1u;                                  // code >= 1 whenever the G bits read one half
    const float h = (float)lo + 0.5f;
    const float mid = lo < r.half ? h * r.inv_grid : __uint_as_float(r.recip_k - __float_as_uint(r.two_m - h));
    const float d = fmaf(-r.s2, mid, ax * r.p);                     // sign(|x| - s * mid), exact
    return (d > 0.0f || (d == 0.0f && (lo & 1u))) ? code : lo;
}

__device__ __forceinline__ uint32_t requant_code(float x, const Requant &r)
{
    const float ax = r.is_signed ? fabsf(x) : fmaxf(x, 0.0f);
    const float q = fminf(ax * r.rinv, r.vmax);
    const float lin = q * r.neg_grid;                                          // -c
    const float rec = __uint_as_float(r.recip_k - __float_as_uint(q));         // 2^m - c
    const float y = q < 1.0f ? lin : rec;
    const uint32_t zb = __float_as_uint(y + __uint_as_float(Requant::kMagic));
    uint32_t code = ((Requant::kRound - zb) >> Requant::G) & r.top;
    if (((zb & ((1u << Requant::G) - 1u)) == (1u << (Requant::G - 1))) | (x != x)) code = requant_settle(x, ax, code, r);
    const uint32_t sign = (__float_as_uint(x) >> r.sign_shift) & r.sign_mask;
    return code ? (code | sign) : 0u;                                          // a zero magnitude never carries the sign
}

// ---- packing across lanes -----------------------------------------------------------------------
// In the matrix-core result layout the 32 lanes of a half-wave hold 32 consecutive columns of one
// row, so the codes of neighbouring lanes are neighbours in the packed row.  Each lane shifts its
// code to its position inside a 32-bit word and the lanes that share the word OR their parts
// together with data-parallel lane permutes (no LDS, no memory); the first lane of the group
// stores the word.  All 64 lanes must be active.
__device__ __forceinline__ uint32_t or_quad(uint32_t w)
{
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0xB1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x4E, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
    return w;
}

// Where a lane's word goes inside the packed row and whether the lane is the one that stores it.
// col = column of the lane's value (a multiple of 32 plus lane % 32).
struct PackSlot {
    uint32_t shift;      // position of the lane's code inside the group's word(s)
    uint32_t byte_off;   // byte offset of the lane's word inside the packed row
    bool stores;
};

__device__ __forceinline__ PackSlot pack_slot(int bits, int lane, uint32_t col)
{
    PackSlot p;
    if (bits == 8) {
        p.shift = (lane & 3) * 8;  p.byte_off = col;            p.stores = (lane & 3) == 0;
    } else if (bits == 4) {
        p.shift = (lane & 7) * 4;  p.byte_off = col >> 1;       p.stores = (lane & 7) == 0;
    } else {                                                    // 6-bit: 16 codes = three words
        const uint32_t k = (lane >> 2) & 3;                     // which group of four inside the 16
        p.shift = (lane & 3) * 6;  p.byte_off = (col >> 4) * 12 + 4 * k;   p.stores = (lane & 3) == 0 && k < 3;
    }
    return p;
}

__device__ __forceinline__ uint32_t pack_word(uint32_t code, int bits, int lane, const PackSlot &p)
{
    uint32_t w = or_quad(code << p.shift);
    if (bits == 4) {
        w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x141, 0xf, 0xf, true);   // row_half_mirror: the other four of eight
    } else if (bits == 6) {
        // four lanes hold 24 bits; word k of the three takes the rest from the next group of four
        const uint32_t k = (lane >> 2) & 3;
        const uint32_t next = (uint32_t)__shfl_down((int)w, 4, 16);
        w = (w >> (8 * k)) | (next << (24 - 8 * k));
    }
    return w;
}

}  // namespace dybit
#endif
