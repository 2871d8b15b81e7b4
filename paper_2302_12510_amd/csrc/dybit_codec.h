// Decoders from packed DyBit codes to fp16 pairs, entirely in the vector ALU (no table look-ups
// in memory).  Shared by the tiled matrix-product kernels.
//
// Every DyBit value of the 2-, 4-, 6- and 8-bit formats is exact in fp16, and so is its 2^-14-fold
// (as a subnormal half below 2^-14), which is what the arithmetic decoders of the 6- and 8-bit
// formats produce: Codec<F>::ACC_EXP is the power of two the epilogue multiplies back in.
// All decoders emit each group
// of eight consecutive k values in the order (k0,k2,k1,k3,k4,k6,k5,k7): that is the order their
// packed arithmetic produces for free, and a contraction does not care about the order of k as
// long as both operands agree.
#ifndef DYBIT_CODEC_H
#define DYBIT_CODEC_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dybit {
namespace fast {

typedef uint32_t u32;
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kOob = 0x80000000u;            // a buffer offset past every supported size: such loads return 0

enum { F4S = 0, F4U = 1, F8S = 2, F8U = 3, F6S = 4, F6U = 5, F2S = 6, F2U = 7 };

// ---------------------------------------------------------------------------
// Codecs: packed codes -> fp16 pairs, entirely in the vector ALU.
// ---------------------------------------------------------------------------
// Arithmetic decoder for m magnitude bits (used for the 6- and 8-bit formats).  With n = 2^m - c
// (1 <= n <= 2^m) held as a half,
//   R = bitcast(K - bits(half(n)))      K = (15 + m) << 10
// is the DyBit value of the code times 2^-14, for every code:
//   * a code with i leading ones, a zero and the k-bit fraction x (k = m-i-1) has n = 2^(k+1) - x, so
//     half(n) has exponent k (k+1 when x == 0) and mantissa 1 - x/2^k; the subtraction turns that into
//     exponent field i and mantissa x/2^k, i.e. 2^(i-1) (1 + x/2^k) 2^-14 (Eq. 1), and its borrow
//     handles x == 0 and the all-ones code (n = 1 -> 2^(m-1) 2^-14);
//   * a code whose first bit is 0 (n > 2^(m-1)) has half(n) in the top binade, the difference has
//     exponent field 0 and mantissa bits c << (11-m): the subnormal half c 2^(1-m) 2^-14, which is
//     the pure fraction of those codes on the same scale (the matrix cores take subnormal halves as
//     they are); c == 0 gives 0.
// The factor 2^14 per arithmetic operand is applied to the accumulators in the epilogue (ACC_EXP);
// it is a power of two, so nothing is rounded differently.
// half(n) comes from the usual trick: the bits 0x6400 | c are the half 1024 + c, and subtracting that
// from 1024 + 2^m leaves n exactly.
__device__ __forceinline__ u32 recip_decode_pair(u32 h, _Float16 base, u32 k2)
{
    const f16x2 nf = (f16x2){base, base} - __builtin_bit_cast(f16x2, h);
    const u16x2 rb = __builtin_bit_cast(u16x2, k2) - __builtin_bit_cast(u16x2, nf);
    return __builtin_bit_cast(u32, rb);
}

// Four 6-bit codes in the low 24 bits of t -> one code per byte (bits above 24 are ignored).
__device__ __forceinline__ u32 unpack_six(u32 t)
{
    return (t & 0x3fu) | ((t << 2) & 0x3f00u) | ((t << 4) & 0x3f0000u) | ((t << 6) & 0x3f000000u);
}

template <int FMT> struct Codec;

// Codec<F>::word decodes one 32-bit word; decode_eight decodes the q-th group of eight codes of
// a thread's 32 codes (held in registers of 128 bits: one for 4-bit codes, two for 8-bit codes,
// the first 24 bytes of two for 6-bit codes, the first 8 bytes of one for 2-bit codes) into four
// registers of two halves.  2- and 6-bit codes: q may run to 7 over a run of 64 codes (one / three registers).
template <int FMT>
__device__ __forceinline__ void decode_eight(const u32x4 *raw, int q, u32 *d)
{
    using C = Codec<FMT>;
    if constexpr (C::BITS == 8) {
        const u32x4 r = raw[q >> 1];
        C::two_words((q & 1) ? r.z : r.x, (q & 1) ? r.w : r.y, d);
    } else if constexpr (C::BITS == 2) {                               // q < 4: a run of 32 codes (8 bytes); q < 8: of 64 codes
        const u32x4 r = raw[0];
        const u32 w = q < 2 ? r.x : q < 4 ? r.y : q < 6 ? r.z : r.w;
        C::half_word((q & 1) ? (w >> 16) : w, d);
    } else if constexpr (C::BITS == 6) {
        // eight codes are 48 bits: two groups of four codes (24 bits) taken out of the run's words (a run of
        // 32 codes is six words, of 64 codes twelve; groups 2 p and 2 p + 1 share words 3 p .. 3 p + 2)
        auto word = [&](int i) -> u32 { const u32x4 r = raw[i >> 2]; return (i & 3) == 0 ? r.x : (i & 3) == 1 ? r.y : (i & 3) == 2 ? r.z : r.w; };
        const int i0 = 3 * (q >> 1);
        u32 ta, tb;
        if ((q & 1) == 0) { ta = word(i0);                                              tb = __builtin_amdgcn_alignbit(word(i0 + 1), word(i0), 24); }
        else              { ta = __builtin_amdgcn_alignbit(word(i0 + 2), word(i0 + 1), 16); tb = word(i0 + 2) >> 8; }
        C::two_words(unpack_six(ta), unpack_six(tb), d);
    } else {
        const u32x4 r = raw[0];
        C::word(q == 0 ? r.x : q == 1 ? r.y : q == 2 ? r.z : r.w, d);
    }
}

// Four independent copies of the arithmetic decoder, written stage by stage so that no
// instruction consumes the result of the one just before it (a packed-fp16 result needs a
// wait state before it can be read).
__device__ __forceinline__ void recip_decode_4pairs(const u32 *h, _Float16 base, u32 k2, u32 *v)
{
    const f16x2 b2 = {base, base};
    f16x2 nf[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) nf[i] = b2 - __builtin_bit_cast(f16x2, h[i]);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = __builtin_bit_cast(u32, __builtin_bit_cast(u16x2, k2) - __builtin_bit_cast(u16x2, nf[i]));
}

template <> struct Codec<F8S> {
    static constexpr int BITS = 8, ACC_EXP = 14;
    // 4 codes (k0..k3) -> (k0,k2), (k1,k3)
    static __device__ __forceinline__ void word(u32 w, u32 *d)
    {
        const u32 wm = w & 0x7f7f7f7fu;                                    // c in every byte
        const u32 h0 = __builtin_amdgcn_perm(0x64646464u, wm, 0x04020400u);
        const u32 h1 = __builtin_amdgcn_perm(0x64646464u, wm, 0x04030401u);
        const u32 v0 = recip_decode_pair(h0, (_Float16)1152.0f, 0x58005800u), v1 = recip_decode_pair(h1, (_Float16)1152.0f, 0x58005800u);
        d[0] = v0 | ((w << 8) & 0x80008000u);                             // sign bit of bytes 0, 2
        d[1] = v1 | (w & 0x80008000u);                                    // sign bit of bytes 1, 3
    }
    // 8 codes (two words) -> four registers, the four pairs decoded side by side
    static __device__ __forceinline__ void two_words(u32 w0, u32 w1, u32 *d)
    {
        const u32 m0 = w0 & 0x7f7f7f7fu, m1 = w1 & 0x7f7f7f7fu;
        u32 h[4], v[4];
        h[0] = __builtin_amdgcn_perm(0x64646464u, m0, 0x04020400u);
        h[1] = __builtin_amdgcn_perm(0x64646464u, m0, 0x04030401u);
        h[2] = __builtin_amdgcn_perm(0x64646464u, m1, 0x04020400u);
        h[3] = __builtin_amdgcn_perm(0x64646464u, m1, 0x04030401u);
        recip_decode_4pairs(h, (_Float16)1152.0f, 0x58005800u, v);
        d[0] = v[0] | ((w0 << 8) & 0x80008000u);
        d[1] = v[1] | (w0 & 0x80008000u);
        d[2] = v[2] | ((w1 << 8) & 0x80008000u);
        d[3] = v[3] | (w1 & 0x80008000u);
    }
};

template <> struct Codec<F8U> {
    static constexpr int BITS = 8, ACC_EXP = 14;
    static __device__ __forceinline__ void word(u32 w, u32 *d)
    {
        const u32 h0 = __builtin_amdgcn_perm(0x64646464u, w, 0x04020400u);
        const u32 h1 = __builtin_amdgcn_perm(0x64646464u, w, 0x04030401u);
        d[0] = recip_decode_pair(h0, (_Float16)1280.0f, 0x5C005C00u);
        d[1] = recip_decode_pair(h1, (_Float16)1280.0f, 0x5C005C00u);
    }
    static __device__ __forceinline__ void two_words(u32 w0, u32 w1, u32 *d)
    {
        u32 h[4];
        h[0] = __builtin_amdgcn_perm(0x64646464u, w0, 0x04020400u);
        h[1] = __builtin_amdgcn_perm(0x64646464u, w0, 0x04030401u);
        h[2] = __builtin_amdgcn_perm(0x64646464u, w1, 0x04020400u);
        h[3] = __builtin_amdgcn_perm(0x64646464u, w1, 0x04030401u);
        recip_decode_4pairs(h, (_Float16)1280.0f, 0x5C005C00u, d);
    }
};

// 6-bit formats: the codes are first spread to one per byte (unpack_six), then the arithmetic
// decoder runs with m = 5 (signed: sign in bit 5 of each byte) or m = 6 magnitude bits.
template <> struct Codec<F6S> {
    static constexpr int BITS = 6, ACC_EXP = 14;
    static __device__ __forceinline__ void two_words(u32 w0, u32 w1, u32 *d)
    {
        const u32 m0 = w0 & 0x1f1f1f1fu, m1 = w1 & 0x1f1f1f1fu;           // c in every byte
        u32 h[4], v[4];
        h[0] = __builtin_amdgcn_perm(0x64646464u, m0, 0x04020400u);
        h[1] = __builtin_amdgcn_perm(0x64646464u, m0, 0x04030401u);
        h[2] = __builtin_amdgcn_perm(0x64646464u, m1, 0x04020400u);
        h[3] = __builtin_amdgcn_perm(0x64646464u, m1, 0x04030401u);
        recip_decode_4pairs(h, (_Float16)1056.0f, 0x50005000u, v);
        d[0] = v[0] | ((w0 << 10) & 0x80008000u);                         // sign: bit 5 of bytes 0, 2
        d[1] = v[1] | ((w0 << 2) & 0x80008000u);                          //       bit 5 of bytes 1, 3
        d[2] = v[2] | ((w1 << 10) & 0x80008000u);
        d[3] = v[3] | ((w1 << 2) & 0x80008000u);
    }
};

template <> struct Codec<F6U> {
    static constexpr int BITS = 6, ACC_EXP = 14;
    static __device__ __forceinline__ void two_words(u32 w0, u32 w1, u32 *d)                  // bytes hold 6 bits each
    {
        u32 h[4];
        h[0] = __builtin_amdgcn_perm(0x64646464u, w0, 0x04020400u);
        h[1] = __builtin_amdgcn_perm(0x64646464u, w0, 0x04030401u);
        h[2] = __builtin_amdgcn_perm(0x64646464u, w1, 0x04020400u);
        h[3] = __builtin_amdgcn_perm(0x64646464u, w1, 0x04030401u);
        recip_decode_4pairs(h, (_Float16)1088.0f, 0x54005400u, d);
    }
};

// 2-bit formats: four values, so the high byte of the half comes from a 4-entry byte table
// (v_perm_b32) indexed by the code itself, sign included; the low byte is zero.
// half_word: 8 codes (k0..k7) in the low 16 bits of w -> (k0,k2), (k1,k3), (k4,k6), (k5,k7).
template <u32 TABLE> struct Codec2 {
    static constexpr int BITS = 2, ACC_EXP = 0;
    static __device__ __forceinline__ u32 spread_even(u32 w)       // fields 0, 2, 4, 6 -> one per byte
    {
        return (w & 0x3u) | ((w << 4) & 0x300u) | ((w << 8) & 0x30000u) | ((w << 12) & 0x3000000u);
    }
    static __device__ __forceinline__ void half_word(u32 w, u32 *d)
    {
        const u32 e = __builtin_amdgcn_perm(0u, TABLE, spread_even(w));         // high bytes of k0 k2 k4 k6
        const u32 o = __builtin_amdgcn_perm(0u, TABLE, spread_even(w >> 2));    // k1 k3 k5 k7
        d[0] = __builtin_amdgcn_perm(0u, e, 0x010c000cu);
        d[1] = __builtin_amdgcn_perm(0u, o, 0x010c000cu);
        d[2] = __builtin_amdgcn_perm(0u, e, 0x030c020cu);
        d[3] = __builtin_amdgcn_perm(0u, o, 0x030c020cu);
    }
};
template <> struct Codec<F2S> : Codec2<0xBC003C00u> {};   // codes 00, 01, 10, 11 -> 0, +1, (-0 =) 0, -1
template <> struct Codec<F2U> : Codec2<0x403C3800u> {};   //                        0, 0.5, 1, 2

// 4-bit formats: every value has at most 3 significant bits, so its half has a zero low byte
// and the high byte comes from an 8-entry byte table held in two registers (v_perm_b32).
template <> struct Codec<F4S> {
    static constexpr int BITS = 4, ACC_EXP = 0;
    // 8 codes (k0..k7) -> (k0,k2), (k1,k3), (k4,k6), (k5,k7)
    static __device__ __forceinline__ void word(u32 w, u32 *d)
    {
        // high bytes of 0, .25, .5, .75, 1, 1.5, 2, 4
        const u32 tlo = 0x3A383400u, thi = 0x44403E3Cu;
        const u32 pe = __builtin_amdgcn_perm(thi, tlo, w & 0x07070707u);           // k0 k2 k4 k6
        const u32 po = __builtin_amdgcn_perm(thi, tlo, (w >> 4) & 0x07070707u);    // k1 k3 k5 k7
        const u32 e = pe | ((w << 4) & 0x80808080u);
        const u32 o = po | (w & 0x80808080u);
        d[0] = __builtin_amdgcn_perm(0u, e, 0x010c000cu);
        d[1] = __builtin_amdgcn_perm(0u, o, 0x010c000cu);
        d[2] = __builtin_amdgcn_perm(0u, e, 0x030c020cu);
        d[3] = __builtin_amdgcn_perm(0u, o, 0x030c020cu);
    }
};

template <> struct Codec<F4U> {
    static constexpr int BITS = 4, ACC_EXP = 0;
    static __device__ __forceinline__ void word(u32 w, u32 *d)
    {
        // high bytes of 0 .. .875 in steps of .125, then 1, 1.25, 1.5, 1.75, 2, 3, 4, 8 (Table I)
        const u32 alo = 0x36343000u, ahi = 0x3B3A3938u, blo = 0x3F3E3D3Cu, bhi = 0x48444240u;
        // two 8-entry byte tables indexed by the low three bits; a third permute takes byte i from the
        // upper table's result where bit 3 of code i is set (selector i + 4), else from the lower one's
        const u32 se = w & 0x07070707u, so = (w >> 4) & 0x07070707u;
        const u32 pick_e = ((w >> 1) & 0x04040404u) | 0x03020100u;
        const u32 pick_o = ((w >> 5) & 0x04040404u) | 0x03020100u;
        const u32 e = __builtin_amdgcn_perm(__builtin_amdgcn_perm(bhi, blo, se), __builtin_amdgcn_perm(ahi, alo, se), pick_e);
        const u32 o = __builtin_amdgcn_perm(__builtin_amdgcn_perm(bhi, blo, so), __builtin_amdgcn_perm(ahi, alo, so), pick_o);
        d[0] = __builtin_amdgcn_perm(0u, e, 0x010c000cu);
        d[1] = __builtin_amdgcn_perm(0u, o, 0x010c000cu);
        d[2] = __builtin_amdgcn_perm(0u, e, 0x030c020cu);
        d[3] = __builtin_amdgcn_perm(0u, o, 0x030c020cu);
    }
};

// A run of 32 codes into registers: one or two 128-bit loads, or (6-bit: 24 bytes, a multiple of 8 from
// the row start) three 64-bit loads, or (2-bit: 8 bytes) one.  An out-of-range offset reads zeros.
template <int BITS>
__device__ __forceinline__ void load_run(const __amdgpu_buffer_rsrc_t rsrc, u32 off, u32x4 *raw)
{
    if constexpr (BITS == 2) {
        const auto a = __builtin_amdgcn_raw_buffer_load_b64(rsrc, off, 0, 0);
        raw[0] = u32x4{a[0], a[1], 0u, 0u};
    } else if constexpr (BITS == 6) {
        const auto a = __builtin_amdgcn_raw_buffer_load_b64(rsrc, off, 0, 0);
        const auto b = __builtin_amdgcn_raw_buffer_load_b64(rsrc, off + 8, 0, 0);
        const auto c = __builtin_amdgcn_raw_buffer_load_b64(rsrc, off + 16, 0, 0);
        raw[0] = u32x4{a[0], a[1], b[0], b[1]};
        raw[1] = u32x4{c[0], c[1], 0u, 0u};
    } else {
#pragma unroll
        for (int p = 0; p < BITS / 4; ++p) raw[p] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off + p * 16, 0, 0);
    }
}

}  // namespace fast
}  // namespace dybit
#endif
