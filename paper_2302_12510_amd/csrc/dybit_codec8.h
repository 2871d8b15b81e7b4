// Decoders from packed 4- and 2-bit DyBit codes to e4m3 bytes for the fp8 matrix path of gfx950
// (`v_mfma_f32_32x32x64_f8f6f4` with both operands e4m3), entirely in the vector ALU.  Every value of the 4-bit
// formats has at most 3 significant bits and lies in [1/8, 8], and the 2-bit formats hold 0, 1/2, 1, 2 or 0, +-1,
// so all are exact in e4m3.  Shared by the tiled kernel (gemm_f8.hip) and the weight-stationary kernel
// (gemm_ws.hip).  The order of the 32 k inside a lane's fragment is the one the 4-bit decoders produce (per eight
// consecutive codes: the four even ones, then the four odd ones); the 2-bit decoders emit the same order, and
// the instruction pairs byte i of an A lane with byte i of the B lane of the same k-quarter.
#ifndef DYBIT_CODEC8_H
#define DYBIT_CODEC8_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dybit_codec.h"

namespace dybit {
namespace f8 {

using namespace fast;

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef u32 u32x2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------
// Decoders: 8 packed 4-bit codes (one word) -> 8 e4m3 bytes in two registers (even codes, odd codes).
// e4m3: sign, 4 exponent bits (bias 7), 3 mantissa bits.
// ---------------------------------------------------------------------------
template <int FMT> struct Codec8;

template <> struct Codec8<F4S> {
    static __device__ __forceinline__ void word(u32 w, u32 *d)
    {
        // e4m3 of 0, .25, .5, .75, 1, 1.5, 2, 4
        const u32 tlo = 0x34302800u, thi = 0x48403C38u;
        const u32 pe = __builtin_amdgcn_perm(thi, tlo, w & 0x07070707u);
        const u32 po = __builtin_amdgcn_perm(thi, tlo, (w >> 4) & 0x07070707u);
        d[0] = pe | ((w << 4) & 0x80808080u);
        d[1] = po | (w & 0x80808080u);
    }
};

template <> struct Codec8<F4U> {
    // e4m3 of 0 .. .875 in steps of .125, then 1, 1.25, 1.5, 1.75, 2, 3, 4, 8 (Table I): two 8-entry byte
    // tables indexed by the low three bits; bit 3 of a code chooses between their results.
    static constexpr u32 alo = 0x2C282000u, ahi = 0x36343230u, blo = 0x3E3C3A38u, bhi = 0x50484440u;
    // The choice as mask arithmetic: 17 instructions per word, short dependency chains (the 256 x 256
    // tile, whose decode hides behind eight MFMAs per fragment, is 1 % faster with this form).
    static __device__ __forceinline__ void word(u32 w, u32 *d)
    {
        const u32 se = w & 0x07070707u, so = (w >> 4) & 0x07070707u;
        const u32 me = w & 0x08080808u, mo = w & 0x80808080u;
        const u32 maske = (me << 5) - (me >> 3), masko = (mo << 1) - (mo >> 7);    // 0xff where bit 3 set
        d[0] = (__builtin_amdgcn_perm(bhi, blo, se) & maske) | (__builtin_amdgcn_perm(ahi, alo, se) & ~maske);
        d[1] = (__builtin_amdgcn_perm(bhi, blo, so) & masko) | (__builtin_amdgcn_perm(ahi, alo, so) & ~masko);
    }
    // The choice as a third permute that takes byte i from the upper table's result where bit 3 of
    // code i is set (selector i + 4) and from the lower one's otherwise (selector i): 13 instructions
    // per word (the smaller tiles, where the decode of A bounds the K loop, are 3 to 6 % faster).
    static __device__ __forceinline__ void word_short(u32 w, u32 *d)
    {
        const u32 se = w & 0x07070707u, so = (w >> 4) & 0x07070707u;
        const u32 pick_e = ((w >> 1) & 0x04040404u) | 0x03020100u;
        const u32 pick_o = ((w >> 5) & 0x04040404u) | 0x03020100u;
        d[0] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(bhi, blo, se), __builtin_amdgcn_perm(ahi, alo, se), pick_e);
        d[1] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(bhi, blo, so), __builtin_amdgcn_perm(ahi, alo, so), pick_o);
    }
};

// 2-bit formats: 16 packed codes (one word) -> 16 e4m3 bytes in four registers, in the order of the
// 4-bit decoders: (k0 k2 k4 k6) (k1 k3 k5 k7) (k8 k10 k12 k14) (k9 k11 k13 k15).  Field j of every
// byte of the word (shift by 2j, mask) gives the codes k = j, j + 4, j + 8, j + 12 as table indices;
// the 4-entry byte table (sign included) is one register, and a second permute puts the bytes of
// fields 0 / 2 (and 1 / 3) side by side.
template <u32 TABLE> struct Codec8Two {
    static __device__ __forceinline__ void word16(u32 w, u32 *d)
    {
        const u32 v0 = __builtin_amdgcn_perm(0u, TABLE, w & 0x03030303u);           // k0 k4 k8 k12
        const u32 v1 = __builtin_amdgcn_perm(0u, TABLE, (w >> 2) & 0x03030303u);    // k1 k5 k9 k13
        const u32 v2 = __builtin_amdgcn_perm(0u, TABLE, (w >> 4) & 0x03030303u);    // k2 k6 k10 k14
        const u32 v3 = __builtin_amdgcn_perm(0u, TABLE, (w >> 6) & 0x03030303u);    // k3 k7 k11 k15
        d[0] = __builtin_amdgcn_perm(v2, v0, 0x05010400u);                          // k0 k2 k4 k6
        d[1] = __builtin_amdgcn_perm(v3, v1, 0x05010400u);
        d[2] = __builtin_amdgcn_perm(v2, v0, 0x07030602u);                          // k8 k10 k12 k14
        d[3] = __builtin_amdgcn_perm(v3, v1, 0x07030602u);
    }
};
template <> struct Codec8<F2S> : Codec8Two<0xB8003800u> {};   // e4m3 of 0, +1, 0 (the unused pattern sign = 1, magnitude = 0), -1
template <> struct Codec8<F2U> : Codec8Two<0x40383000u> {};   // e4m3 of 0, 0.5, 1, 2

template <int FMT> constexpr int bits_of() { return (FMT == F2S || FMT == F2U) ? 2 : 4; }

// 32 codes -> one 32-byte fragment.  4-bit: the four words of r; 2-bit: words `first`, `first + 1`.
// SHORT: the variant of the decoder with fewer instructions, where a format has two.
template <int FMT, bool SHORT = false>
__device__ __forceinline__ i32x8 decode_fragment(const u32x4 r, int first = 0)
{
    u32 d[8];
    if constexpr (bits_of<FMT>() == 2) {
        Codec8<FMT>::word16(first ? r.z : r.x, d);
        Codec8<FMT>::word16(first ? r.w : r.y, d + 4);
    } else if constexpr (FMT == F4U && SHORT) {
        Codec8<FMT>::word_short(r.x, d);
        Codec8<FMT>::word_short(r.y, d + 2);
        Codec8<FMT>::word_short(r.z, d + 4);
        Codec8<FMT>::word_short(r.w, d + 6);
    } else {
        Codec8<FMT>::word(r.x, d);
        Codec8<FMT>::word(r.y, d + 2);
        Codec8<FMT>::word(r.z, d + 4);
        Codec8<FMT>::word(r.w, d + 6);
    }
    return i32x8{(int)d[0], (int)d[1], (int)d[2], (int)d[3], (int)d[4], (int)d[5], (int)d[6], (int)d[7]};
}

}  // namespace f8
}  // namespace dybit
#endif
