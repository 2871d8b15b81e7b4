// Large-tile DyBit matrix product for gfx950: 256 x 256 tile of C per workgroup, K step 64,
// four waves (one per SIMD) each owning 128 x 128 of C in 256 accumulator registers.
//
// Data path per K step: packed codes come from HBM/L2 with 128-bit buffer loads (two steps
// ahead), are decoded to fp16 in the vector ALU (no table look-ups: see the codecs below),
// written once to a double-buffered, XOR-swizzled LDS tile and read back as MFMA fragments by
// the waves that need them.  The decode of step t+1 is interleaved with the 64 MFMAs of step t.
//
// The order of k inside one MFMA does not matter as long as both operands agree, so both
// codecs emit each group of eight k values in the order (k0,k2,k1,k3,k4,k6,k5,k7): that is
// the order in which their packed arithmetic produces them for free.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <type_traits>

#include "gemm_args.h"

namespace dybit {
namespace fast {

typedef uint32_t u32;
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));

constexpr int TM = 256, TN = 256, TK = 64;
constexpr int THREADS = 256;
constexpr int ROW_BYTES = TK * 2 + 16;            // one LDS row: 64 halves = 8 chunks of 16 B, plus 16 B of padding
constexpr int STAGE_BYTES = TM * ROW_BYTES;       // 36 KiB per operand per stage
constexpr int LDS_BYTES = 4 * STAGE_BYTES;        // A0 A1 W0 W1
constexpr uint32_t kOob = 0x80000000u;            // a buffer offset past every supported size: such loads return 0

enum { F4S = 0, F4U = 1, F8S = 2, F8U = 3 };

// ---------------------------------------------------------------------------
// Codecs: packed codes -> fp16 pairs, entirely in the vector ALU.
// ---------------------------------------------------------------------------
// Arithmetic decoder for m magnitude bits (used for the 8-bit formats).  With n = 2^m - c:
//   R = bitcast(K - bits(half(n)))      K = (15 + 15 + m-1) << 10
// equals the DyBit value for codes with a leading one (see magnitude_value in dybit_device.h),
// and for codes below that (n >= 2^(m-1)) it equals 1/2 + c/2^m, so the fraction c/2^(m-1) is
// 2R - 1.  Because 2R - 1 >= R exactly when R >= 1, the value is min(R, 2R - 1) for every code.
// half(n) comes from the usual trick: the bits 0x6400 | (2^m - 1 - c) are the half 1024 + 2^m-1-c,
// and subtracting 1023 leaves n.  Both R and 2R-1 are non-negative, so the minimum is taken
// on the bit patterns (no NaN canonicalisation needed).
__device__ __forceinline__ u32 recip_decode_pair(u32 h, u32 k2)
{
    const f16x2 nf = __builtin_bit_cast(f16x2, h) + (f16x2){(_Float16)-1023.0f, (_Float16)-1023.0f};
    const u16x2 rb = __builtin_bit_cast(u16x2, k2) - __builtin_bit_cast(u16x2, nf);
    const f16x2 R = __builtin_bit_cast(f16x2, rb);
    const f16x2 L = R * (f16x2){(_Float16)2.0f, (_Float16)2.0f} + (f16x2){(_Float16)-1.0f, (_Float16)-1.0f};
    const u16x2 v = __builtin_elementwise_min(rb, __builtin_bit_cast(u16x2, L));
    return __builtin_bit_cast(u32, v);
}

template <int FMT> struct Codec;

template <> struct Codec<F8S> {
    static constexpr int BITS = 8;
    // 4 codes (k0..k3) -> (k0,k2), (k1,k3)
    static __device__ __forceinline__ void word(u32 w, u32 *d)
    {
        const u32 wm = ~w & 0x7f7f7f7fu;                                   // 127 - c in every byte
        const u32 h0 = __builtin_amdgcn_perm(0x64646464u, wm, 0x04020400u);
        const u32 h1 = __builtin_amdgcn_perm(0x64646464u, wm, 0x04030401u);
        const u32 v0 = recip_decode_pair(h0, 0x90009000u), v1 = recip_decode_pair(h1, 0x90009000u);
        d[0] = (v0 & 0x7fff7fffu) | ((w << 8) & 0x80008000u);             // sign bit of bytes 0, 2
        d[1] = (v1 & 0x7fff7fffu) | (w & 0x80008000u);                    // sign bit of bytes 1, 3
    }
};

template <> struct Codec<F8U> {
    static constexpr int BITS = 8;
    static __device__ __forceinline__ void word(u32 w, u32 *d)
    {
        const u32 wm = ~w;                                                 // 255 - c in every byte
        const u32 h0 = __builtin_amdgcn_perm(0x64646464u, wm, 0x04020400u);
        const u32 h1 = __builtin_amdgcn_perm(0x64646464u, wm, 0x04030401u);
        d[0] = recip_decode_pair(h0, 0x94009400u);
        d[1] = recip_decode_pair(h1, 0x94009400u);
    }
};

// 4-bit formats: every value has at most 3 significant bits, so its half has a zero low byte
// and the high byte comes from an 8-entry byte table held in two registers (v_perm_b32).
template <> struct Codec<F4S> {
    static constexpr int BITS = 4;
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
    static constexpr int BITS = 4;
    static __device__ __forceinline__ void word(u32 w, u32 *d)
    {
        // high bytes of 0 .. .875 in steps of .125, then 1, 1.25, 1.5, 1.75, 2, 3, 4, 8 (Table I)
        const u32 alo = 0x36343000u, ahi = 0x3B3A3938u, blo = 0x3F3E3D3Cu, bhi = 0x48444240u;
        const u32 se = w & 0x07070707u, so = (w >> 4) & 0x07070707u;
        const u32 me = w & 0x08080808u, mo = w & 0x80808080u;
        const u32 maske = (me << 5) - (me >> 3), masko = (mo << 1) - (mo >> 7);    // 0xff where bit 3 set
        const u32 e = (__builtin_amdgcn_perm(bhi, blo, se) & maske) | (__builtin_amdgcn_perm(ahi, alo, se) & ~maske);
        const u32 o = (__builtin_amdgcn_perm(bhi, blo, so) & masko) | (__builtin_amdgcn_perm(ahi, alo, so) & ~masko);
        d[0] = __builtin_amdgcn_perm(0u, e, 0x010c000cu);
        d[1] = __builtin_amdgcn_perm(0u, o, 0x010c000cu);
        d[2] = __builtin_amdgcn_perm(0u, e, 0x030c020cu);
        d[3] = __builtin_amdgcn_perm(0u, o, 0x030c020cu);
    }
};

// ---------------------------------------------------------------------------
// Per-thread staging of one operand tile (256 rows x 64 codes).
//   8-bit: 4 loads of 16 B; load j covers row t/4 + 64 j, codes 16 s .. 16 s + 15 (s = t % 4)
//          and decodes to LDS chunks 2 s and 2 s + 1 of that row.
//   4-bit: 2 loads of 16 B; load j covers row t/2 + 128 j, codes 32 s .. 32 s + 31 (s = t % 2)
//          and decodes to LDS chunks 4 s .. 4 s + 3.
// LDS chunk c of row r sits at r * 144 + c * 16: the 16 B of padding rotate the banks by one
// chunk per row, so fragment reads (32 consecutive rows, same chunk) and these writes are both
// free of bank conflicts, and every address is one base register plus an immediate.
// ---------------------------------------------------------------------------
template <int BITS> struct Staging {
    static constexpr int NLOAD = BITS == 8 ? 4 : 2;
    static constexpr int ROWS_PER_LOAD = TM / NLOAD;
    static constexpr int TPR = THREADS / ROWS_PER_LOAD;          // threads per row: 4 or 2
    static constexpr int TILE_K_BYTES = TK * BITS / 8;           // 64 or 32
    static constexpr int CHUNKS = 8 / TPR;                       // chunks written per load: 2 or 4
};

template <int FMT>
__device__ __forceinline__ void decode_quarter(const u32x4 *raw, int quarter, char *lds_tile, u32 wr_base)
{
    using C = Codec<FMT>;
    using S = Staging<C::BITS>;
    // wr_base: byte address of the first chunk this thread writes in the row of load 0
    u32 d[8];
    u32 off;
    if (C::BITS == 8) {
        const u32x4 r = raw[quarter];
        C::word(r.x, d); C::word(r.y, d + 2); C::word(r.z, d + 4); C::word(r.w, d + 6);
        off = quarter * S::ROWS_PER_LOAD * ROW_BYTES;
    } else {
        const u32x4 r = raw[quarter >> 1];
        C::word((quarter & 1) ? r.z : r.x, d); C::word((quarter & 1) ? r.w : r.y, d + 4);
        off = (quarter >> 1) * S::ROWS_PER_LOAD * ROW_BYTES + (quarter & 1) * 32;
    }
    *reinterpret_cast<u32x4 *>(lds_tile + wr_base + off) = u32x4{d[0], d[1], d[2], d[3]};
    *reinterpret_cast<u32x4 *>(lds_tile + wr_base + off + 16) = u32x4{d[4], d[5], d[6], d[7]};
}

template <int FMT_A, int FMT_W, bool CONV>
__global__ __launch_bounds__(THREADS) void gemm_fast_kernel(const GemmArgs g, const int tiles_m, const int tiles_n)
{
    using CA = Codec<FMT_A>;
    using CW = Codec<FMT_W>;
    using SA = Staging<CA::BITS>;
    using SW = Staging<CW::BITS>;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char *const ldsA = lds, *const ldsW = lds + 2 * STAGE_BYTES;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- tile assignment: consecutive workgroup ids go to different XCDs (8 of them); give
    // each XCD a compact 4 x 8 patch of the 16 x 16-tile region that is in flight, so that the
    // A and W strips it streams are shared inside its own L2.
    int tile_m, tile_n;
    {
        const int b = blockIdx.x;
        const int per_region = 256;
        const int region = b / per_region, r = b % per_region;
        const int xcd = r & 7, i = r >> 3;                         // i: 0..31 inside the XCD
        const int regions_n = (tiles_n + 15) / 16;
        const int rm = region / regions_n, rn = region % regions_n;
        tile_m = rm * 16 + (xcd >> 1) * 4 + (i >> 3);
        tile_n = rn * 16 + (xcd & 1) * 8 + (i & 7);
        if (tile_m >= tiles_m || tile_n >= tiles_n) return;       // uniform per workgroup
    }
    const int64_t m0 = (int64_t)tile_m * TM, n0 = (int64_t)tile_n * TN;

    const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(g.A), 0, (int)(g.a_bytes > 0x7fffffff ? 0x7fffffff : g.a_bytes), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(g.W), 0, (int)(g.w_bytes > 0x7fffffff ? 0x7fffffff : g.w_bytes), 0x00020000);

    // ---- per-thread load descriptors
    const int a_row_bytes = (int)(g.K * CA::BITS / 8), w_row_bytes = (int)(g.K * CW::BITS / 8);
    const int pix_bytes = CONV ? g.Cin * CA::BITS / 8 : 0;
    u32 offA[SA::NLOAD];
    int hi0[SA::NLOAD], wi0[SA::NLOAD];
    bool okA[SA::NLOAD];
#pragma unroll
    for (int j = 0; j < SA::NLOAD; ++j) {
        const int64_t m = m0 + tid / SA::TPR + j * SA::ROWS_PER_LOAD;
        okA[j] = m < g.M;
        const int seg = (tid % SA::TPR) * 16;
        if (CONV) {
            const int64_t mm = okA[j] ? m : 0;
            const int b = (int)(mm / ((int64_t)g.Ho * g.Wo));
            const int rem = (int)(mm - (int64_t)b * g.Ho * g.Wo);
            const int ho = rem / g.Wo, wo = rem - ho * g.Wo;
            hi0[j] = ho * g.stride - g.pad;
            wi0[j] = wo * g.stride - g.pad;
            offA[j] = (u32)((((int64_t)b * g.H + hi0[j]) * g.Wd + wi0[j]) * pix_bytes + seg);
        } else {
            hi0[j] = wi0[j] = 0;
            offA[j] = okA[j] ? (u32)(m * a_row_bytes + seg) : kOob;
        }
    }
    u32 offW[SW::NLOAD];
#pragma unroll
    for (int j = 0; j < SW::NLOAD; ++j) {
        const int64_t n = n0 + tid / SW::TPR + j * SW::ROWS_PER_LOAD;
        offW[j] = n < g.N ? (u32)(n * w_row_bytes + (tid % SW::TPR) * 16) : kOob;
    }

    auto load_tile = [&](int64_t kt, u32x4 *rawA, u32x4 *rawW) {
        const int64_t k0 = kt * TK;
        if (CONV) {
            const int tap = (int)(k0 / g.Cin), c0 = (int)(k0 - (int64_t)tap * g.Cin);    // uniform
            const int fr = tap / g.kw, fs = tap - fr * g.kw;
            const int tap_off = (fr * g.Wd + fs) * pix_bytes + c0 * CA::BITS / 8;
#pragma unroll
            for (int j = 0; j < SA::NLOAD; ++j) {
                const bool in = okA[j] && (unsigned)(hi0[j] + fr) < (unsigned)g.H && (unsigned)(wi0[j] + fs) < (unsigned)g.Wd;
                const u32 off = in ? offA[j] + (u32)tap_off : kOob;            // out of range reads 0 = code 0
                rawA[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, off, 0, 0);
            }
        } else {
            // rows past M start at kOob and stay out of range while k advances
            const u32 koff = (u32)(k0 * CA::BITS / 8);
#pragma unroll
            for (int j = 0; j < SA::NLOAD; ++j) rawA[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, offA[j] + koff, 0, 0);
        }
        const u32 koffw = (u32)(k0 * CW::BITS / 8);
#pragma unroll
        for (int j = 0; j < SW::NLOAD; ++j) rawW[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrcW, offW[j] + koffw, 0, 0);
    };

    // ---- LDS addresses
    const u32 wrA = (u32)(tid / SA::TPR) * ROW_BYTES + (u32)(tid % SA::TPR) * (128 / SA::TPR);
    const u32 wrW = (u32)(tid / SW::TPR) * ROW_BYTES + (u32)(tid % SW::TPR) * (128 / SW::TPR);
    // fragment reads: row (lane & 31) of a 32-row block, chunk 2 kk + (lane >> 5)
    const u32 rdA = (u32)(wm * 128 + (lane & 31)) * ROW_BYTES + (u32)(lane >> 5) * 16;
    const u32 rdW = (u32)(wn * 128 + (lane & 31)) * ROW_BYTES + (u32)(lane >> 5) * 16;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int64_t ktiles = g.K / TK;
    u32x4 rawA[2][SA::NLOAD], rawW[2][SW::NLOAD];

    // ---- prologue: tile 0 decoded into stage 0, tile 1 in flight, fragments of k block 0 in registers
    load_tile(0, rawA[0], rawW[0]);
    if (ktiles > 1) load_tile(1, rawA[1], rawW[1]);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        decode_quarter<FMT_A>(rawA[0], q, ldsA, wrA);
        decode_quarter<FMT_W>(rawW[0], q, ldsW, wrW);
    }
    __syncthreads();

    f16x8 fa[2][4], fw[2][4];
    auto read_frags = [&](const char *tileA, const char *tileW, int kk, int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) fa[buf][i] = *reinterpret_cast<const f16x8 *>(tileA + rdA + kk * 32 + i * 32 * ROW_BYTES);
#pragma unroll
        for (int j = 0; j < 4; ++j) fw[buf][j] = *reinterpret_cast<const f16x8 *>(tileW + rdW + kk * 32 + j * 32 * ROW_BYTES);
    };
    read_frags(ldsA, ldsW, 0, 0);

    // One K step over LDS stage s.  Four k blocks of 16 MFMAs each; the fragments of a block are
    // read one block ahead.  The next tile is decoded into the other stage during blocks 0..2,
    // the workgroup barrier sits before block 3, and the first fragments of the next tile are
    // requested right after it, so that their LDS latency hides behind the MFMAs of block 3.
    //   MODE 2: decode the next tile and load the one after;  1: decode only;  0: last tile.
    auto step = [&](int64_t kt, auto stage_tag, auto mode_tag) {
        constexpr int s = decltype(stage_tag)::value;
        constexpr int MODE = decltype(mode_tag)::value;
        const char *curA = ldsA + s * STAGE_BYTES, *curW = ldsW + s * STAGE_BYTES;
        char *nxtA = ldsA + (s ^ 1) * STAGE_BYTES, *nxtW = ldsW + (s ^ 1) * STAGE_BYTES;
        if (MODE == 2) load_tile(kt + 2, rawA[s], rawW[s]);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int cb = kk & 1, nb = cb ^ 1;
            if (kk == 3 && MODE >= 1) {
                __syncthreads();
                read_frags(nxtA, nxtW, 0, nb);
            } else if (kk < 3) {
                read_frags(curA, curW, kk + 1, nb);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[cb][i], fw[cb][j], acc[i][j], 0, 0, 0);
            if (MODE >= 1 && kk < 3) {
                // decode work of the next tile, spread over blocks 0..2 in three near-equal parts
                if (kk == 0) {
                    decode_quarter<FMT_A>(rawA[s ^ 1], 0, nxtA, wrA);
                    decode_quarter<FMT_W>(rawW[s ^ 1], 0, nxtW, wrW);
                    decode_quarter<FMT_W>(rawW[s ^ 1], 1, nxtW, wrW);
                } else if (kk == 1) {
                    decode_quarter<FMT_A>(rawA[s ^ 1], 1, nxtA, wrA);
                    decode_quarter<FMT_A>(rawA[s ^ 1], 2, nxtA, wrA);
                } else {
                    decode_quarter<FMT_A>(rawA[s ^ 1], 3, nxtA, wrA);
                    decode_quarter<FMT_W>(rawW[s ^ 1], 2, nxtW, wrW);
                    decode_quarter<FMT_W>(rawW[s ^ 1], 3, nxtW, wrW);
                }
            }
            // Order inside the block: the eight fragment reads first, then MFMAs with the decode
            // arithmetic between them, the tile writes towards the end.
            __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);                     // DS read x 8
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // MFMA
                if (MODE >= 1 && kk < 3) __builtin_amdgcn_sched_group_barrier(0x002, 7, 0);   // VALU
                if (MODE >= 1 && kk < 3 && r >= 3 && (r & 1)) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // DS write
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using T0 = std::integral_constant<int, 0>;
    using T1 = std::integral_constant<int, 1>;
    using M0 = std::integral_constant<int, 0>;
    using M1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;

    // tiles 0 .. ktiles-3 in MODE 2, tile ktiles-2 in MODE 1, tile ktiles-1 in MODE 0
    int64_t kt = 0;
    for (; kt + 3 < ktiles; kt += 2) {
        step(kt, T0{}, M2{});
        step(kt + 1, T1{}, M2{});
    }
    if (kt + 3 == ktiles) {
        step(kt, T0{}, M2{});
        step(kt + 1, T1{}, M1{});
        step(kt + 2, T0{}, M0{});
    } else if (kt + 2 == ktiles) {
        step(kt, T0{}, M1{});
        step(kt + 1, T1{}, M0{});
    } else {
        step(kt, T0{}, M0{});
    }

    // ---- epilogue: C = acc * (sA sW) (+ bias) (ReLU).  Accumulator v of a lane is row
    // 8 (v / 4) + 4 (lane / 32) + v % 4 and column lane % 32 of its 32 x 32 block.
    const float alpha = (*g.a_scale) * (*g.w_scale);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t n = n0 + wn * 128 + j * 32 + (lane & 31);
        const bool n_ok = n < g.N;
        const float b = (g.bias && n_ok) ? g.bias[n] : 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t m = m0 + wm * 128 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                float c = acc[i][j][v] * alpha + b;
                if (g.relu) c = fmaxf(c, 0.0f);
                if (n_ok && m < g.M) __builtin_nontemporal_store(c, g.C + m * g.ldc + n);
            }
        }
    }
}

template <int FA, int FW>
static void launch(const GemmArgs &g, bool conv, hipStream_t st)
{
    const int tiles_m = (int)((g.M + TM - 1) / TM), tiles_n = (int)((g.N + TN - 1) / TN);
    const int regions = ((tiles_m + 15) / 16) * ((tiles_n + 15) / 16);
    const dim3 grid(regions * 256), block(THREADS);
    if (conv) {
        auto k = gemm_fast_kernel<FA, FW, true>;
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        hipLaunchKernelGGL(k, grid, block, LDS_BYTES, st, g, tiles_m, tiles_n);
    } else {
        auto k = gemm_fast_kernel<FA, FW, false>;
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        hipLaunchKernelGGL(k, grid, block, LDS_BYTES, st, g, tiles_m, tiles_n);
    }
}

}  // namespace fast

bool launch_gemm_fast(const GemmArgs &g, int a_bits, int w_bits, bool conv, hipStream_t st)
{
    using namespace fast;
    if ((a_bits != 4 && a_bits != 8) || (w_bits != 4 && w_bits != 8)) return false;
    if (g.K < TK || g.K % TK) return false;
    if (conv && g.Cin % TK) return false;                                  // a K step must stay inside one filter tap
    if ((reinterpret_cast<uintptr_t>(g.A) | reinterpret_cast<uintptr_t>(g.W)) & 15) return false;
    // 32-bit buffer offsets, including the rows past M / N that the last tiles touch
    if (g.a_bytes + (int64_t)TM * g.K * a_bits / 8 >= 0x7fffffff || g.w_bytes + (int64_t)TN * g.K * w_bits / 8 >= 0x7fffffff) return false;
    // Too few large tiles cannot fill 256 compute units; DYBIT_FAST_MIN_TILES overrides the
    // threshold (tests use it to reach this kernel with small shapes).
    const char *env = getenv("DYBIT_FAST_MIN_TILES");
    const int64_t min_tiles = env ? atoll(env) : 128;
    if (((g.M + TM - 1) / TM) * ((g.N + TN - 1) / TN) < min_tiles) return false;
    const int fa = (a_bits == 8 ? F8S : F4S) + (g.a_signed ? 0 : 1);
    const int fw = (w_bits == 8 ? F8S : F4S) + (g.w_signed ? 0 : 1);
#define DYBIT_F(A_, W_) case (A_) * 4 + (W_): launch<A_, W_>(g, conv, st); return true
    switch (fa * 4 + fw) {
        DYBIT_F(F8S, F4S);
        DYBIT_F(F4U, F4S);
        default: return false;
    }
#undef DYBIT_F
}

}  // namespace dybit
