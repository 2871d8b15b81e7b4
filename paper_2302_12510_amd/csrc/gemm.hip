// DyBit x DyBit matrix product and implicit-GEMM convolution for gfx950 (MFMA, fp32 accumulate).
//
// Every DyBit value of every supported format is exactly representable in IEEE half precision
// (at most 7 significant bits, magnitudes 2^-7 .. 2^7), so both operands are decoded to fp16 and
// multiplied with v_mfma_f32_32x32x16_f16: the products are exact and only the fp32
// accumulation rounds.  This file holds the C entry points and the general kernel (any format
// pair, any shape): packed codes are streamed from HBM, decoded through a per-operand lookup
// table that lives in LDS, staged in LDS as fp16 tiles and consumed by the matrix cores.  Large
// 4/8-bit problems are routed to the large-tile kernel of gemm_fast.hip first.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dybit_device.h"
#include "dybit_host.h"
#include "gemm_args.h"
#include "tile_epilogue.h"

namespace dybit {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// General kernel: any format pair, any shape.
// ---------------------------------------------------------------------------
constexpr int BM = 128, BN = 128, BK = 64;     // tile of C and the K step, in elements
constexpr int LDK = BK + 8;                    // LDS row pitch in halves (144 B: conflict-free b128 reads)
constexpr int GEMM_THREADS = 256;              // 4 waves, 2 x 2, each 64 x 64 of C
constexpr int UNIT = 16;                       // elements decoded at a time (one run along K)

// A "unit" is 16 consecutive codes of one row, held in registers exactly as they are packed in
// memory: 16 B (8-bit), 12 B (6-bit), 8 B (4-bit) or 4 B (2-bit).
template <int BITS> struct Unit { uint32_t w[BITS / 2]; };

// Lookup tables (32-bit entries).  8- and 6-bit: indexed by the code, low half = fp16 value.
// 4-bit: indexed by a packed byte, two fp16 values (low nibble first).  2-bit: indexed by a
// nibble (two codes), two fp16 values.
template <int BITS> constexpr int lut_entries() { return BITS == 8 ? 256 : BITS == 6 ? 64 : BITS == 4 ? 256 : 16; }

__device__ __forceinline__ uint32_t half_bits(float v)
{
    const _Float16 h = (_Float16)v;            // exact for every DyBit value
    return (uint32_t) __builtin_bit_cast(uint16_t, h);
}

template <int BITS>
__device__ __forceinline__ void build_lut(uint32_t *lut, int is_signed, int tid)
{
    for (int e = tid; e < lut_entries<BITS>(); e += GEMM_THREADS) {
        uint32_t v;
        if (BITS == 8 || BITS == 6) {
            v = half_bits(code_value(e, BITS, is_signed));
        } else {
            const uint32_t lo = e & ((1u << BITS) - 1), hi = (e >> BITS) & ((1u << BITS) - 1);
            v = half_bits(code_value(lo, BITS, is_signed)) | (half_bits(code_value(hi, BITS, is_signed)) << 16);
        }
        lut[e] = v;
    }
}

// 16 codes -> 16 halves (two 128-bit vectors), in K order.
template <int BITS>
__device__ __forceinline__ void decode_unit(const Unit<BITS> &u, const uint32_t *lut, u32x4 &lo, u32x4 &hi)
{
    uint32_t h[8];
    if (BITS == 8) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t w = u.w[j >> 1] >> ((j & 1) * 16);
            h[j] = (lut[w & 0xff] & 0xffffu) | (lut[(w >> 8) & 0xff] << 16);
        }
    } else if (BITS == 4) {
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = lut[(u.w[j >> 2] >> ((j & 3) * 8)) & 0xff];
    } else if (BITS == 2) {
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = lut[(u.w[0] >> (j * 4)) & 0xf];
    } else {  // 6-bit: 96-bit stream
        const uint64_t s0 = (uint64_t)u.w[0] | ((uint64_t)u.w[1] << 32);        // bits 0..63
        const uint64_t s1 = (uint64_t)u.w[1] | ((uint64_t)u.w[2] << 32);        // bits 32..95
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t c[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int bit = 6 * (2 * j + t);
                c[t] = (bit + 6 <= 64) ? (uint32_t)(s0 >> bit) & 63u : (uint32_t)(s1 >> (bit - 32)) & 63u;
            }
            h[j] = (lut[c[0]] & 0xffffu) | (lut[c[1]] << 16);
        }
    }
    lo = u32x4{h[0], h[1], h[2], h[3]};
    hi = u32x4{h[4], h[5], h[6], h[7]};
}

// One code of a packed row (bounds are the caller's business).
template <int BITS>
__device__ __forceinline__ uint32_t fetch_code(const uint8_t *row, int64_t k)
{
    const int64_t bit = k * BITS;
    uint32_t w = row[bit >> 3];
    // a 6-bit code that starts past bit 2 of its byte continues in the next one; otherwise the same
    // byte is read again (its copy lands above the field and is masked off): no branch, no read
    // past the code's own bytes
    if (BITS == 6) w |= (uint32_t)row[(bit >> 3) + ((bit & 7) > 2 ? 1 : 0)] << 8;
    return (w >> (bit & 7)) & ((1u << BITS) - 1);
}

template <int BITS>
__device__ __forceinline__ void unit_set_code(Unit<BITS> &u, int e, uint32_t c)
{
    const int bit = e * BITS;
    u.w[bit >> 5] |= c << (bit & 31);
    if (BITS == 6 && (bit & 31) > 26) u.w[(bit >> 5) + 1] |= c >> (32 - (bit & 31));
}

template <int BITS>
__device__ __forceinline__ Unit<BITS> load_unit_vec(const uint8_t *p)
{
    Unit<BITS> u;
    if (BITS == 8) {
        const u32x4 v = *reinterpret_cast<const u32x4 *>(p);
        u.w[0] = v.x; u.w[1] = v.y; u.w[2] = v.z; u.w[3] = v.w;
    } else if (BITS == 4) {
        const uint2 v = *reinterpret_cast<const uint2 *>(p);
        u.w[0] = v.x; u.w[1] = v.y;
    } else if (BITS == 6) {
        const uint32_t *q = reinterpret_cast<const uint32_t *>(p);
        u.w[0] = q[0]; u.w[1] = q[1]; u.w[2] = q[2];
    } else {
        u.w[0] = *reinterpret_cast<const uint32_t *>(p);
    }
    return u;
}

// 16 consecutive codes of a packed row fetched one by one (rows whose length or alignment rules
// out vector loads); codes past K read as 0.  Every fetch is issued before any is used.
template <int BITS>
__device__ __forceinline__ Unit<BITS> load_unit_elems(const uint8_t *row, int64_t k0, int64_t K)
{
    Unit<BITS> u;
#pragma unroll
    for (int i = 0; i < BITS / 2; ++i) u.w[i] = 0;
    uint32_t code[UNIT];
#pragma unroll
    for (int e = 0; e < UNIT; ++e) {
        const bool in = k0 + e < K;
        const uint32_t v = fetch_code<BITS>(row, in ? k0 + e : k0);
        code[e] = in ? v : 0u;
    }
#pragma unroll
    for (int e = 0; e < UNIT; ++e) unit_set_code<BITS>(u, e, code[e]);
    return u;
}

// Row descriptor of the activation operand: a plain matrix row, or an output pixel of a convolution.
struct RowA {
    const uint8_t *base;   // GEMM: start of the row; CONV: start of image b
    uint32_t img_off;      // CONV: byte offset of image b inside the activation tensor
    int hi0, wi0;          // CONV: top-left input coordinate of the receptive field
    bool valid;
};

// How the kernel reaches its operands.
//   ELEMS  code by code: any K, any Cin, any alignment
//   VEC    a 16-code unit is one aligned vector load (GEMM: K, convolution: Cin a multiple of 16)
//   RUNS   convolution with few channels (Cin divides 16, kw * Cin a multiple of 16): a unit is
//          16 / Cin neighbouring taps of one filter row, which are contiguous in the image; weights
//          as in VEC (K is then a multiple of 16)
enum : int { ELEMS = 0, VEC = 1, RUNS = 2 };

// RUNS: 16 codes = `taps` pixels starting at filter row fr, tap ur * taps.  The run starts at any
// byte, so it is fetched as aligned words through a buffer descriptor (words before the tensor or
// past its end read 0) and shifted into place; taps left or right of the image are masked to code
// 0, a filter row above or below it reads nothing.
template <int BITS>
__device__ __forceinline__ Unit<BITS> load_unit_A_run(const GemmArgs &g, const __amdgpu_buffer_rsrc_t rsrc, const RowA &r,
                                                      int fr, int ur, int64_t k0)
{
    constexpr int NWORD = BITS / 2;
    Unit<BITS> u;
    const int taps = UNIT / g.Cin, tap_bits = g.Cin * BITS;
    const int hi = r.hi0 + fr, wi = r.wi0 + ur * taps;
    const bool row_ok = r.valid && k0 < g.K && (unsigned)hi < (unsigned)g.H;
    const int byte_off = (int)r.img_off + (hi * g.Wd + wi) * (tap_bits / 8);   // negative left of the first pixel
    const int shift = byte_off & 3;
    const int base = byte_off - shift;
    uint32_t raw[NWORD + 1];
#pragma unroll
    for (int j = 0; j <= NWORD; ++j) {
        // a word before the tensor gets the out-of-range offset explicitly: the hardware adds offsets
        // without wrapping at 32 bits, so a negative offset plus 4 j would not come back into range
        const int o = base + 4 * j;
        raw[j] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, (row_ok && o >= 0) ? (uint32_t)o : 0x80000000u, 0, 0);
    }
    int t_lo = max(0, -wi), t_hi = min(taps, g.Wd - wi);
    t_hi = max(t_hi, t_lo);
    const int bit_lo = t_lo * tap_bits, bit_hi = t_hi * tap_bits;
#pragma unroll
    for (int i = 0; i < NWORD; ++i) {
        const int lo = min(max(bit_lo - 32 * i, 0), 32), up = min(max(bit_hi - 32 * i, 0), 32);
        const uint32_t keep = (uint32_t)((1ull << up) - 1ull) & ~(uint32_t)((1ull << lo) - 1ull);
        u.w[i] = __builtin_amdgcn_alignbyte(raw[i + 1], raw[i], (uint32_t)shift) & keep;
    }
    return u;
}

template <int BITS, bool CONV, int MODE>
__device__ __forceinline__ Unit<BITS> load_unit_A(const GemmArgs &g, const RowA &r, int64_t k0)
{
    Unit<BITS> u;
#pragma unroll
    for (int i = 0; i < BITS / 2; ++i) u.w[i] = 0;
    if (!r.valid || k0 >= g.K) return u;
    if (!CONV) {
        if (MODE == VEC) return load_unit_vec<BITS>(r.base + k0 * BITS / 8);
        return load_unit_elems<BITS>(r.base, k0, g.K);
    }
    const int64_t pix_bytes = g.pix_bytes;
    if (MODE == VEC) {   // the whole unit lies inside one filter tap
        const int tap = (int)(k0 / g.Cin), c0 = (int)(k0 - (int64_t)tap * g.Cin);
        const int fr = tap / g.kw, fs = tap - fr * g.kw;
        const int hi = r.hi0 + fr, wi = r.wi0 + fs;
        if (hi < 0 || hi >= g.H || wi < 0 || wi >= g.Wd) return u;       // padding: code 0 = 0.0
        return load_unit_vec<BITS>(r.base + ((int64_t)hi * g.Wd + wi) * pix_bytes + (int64_t)c0 * BITS / 8);
    }
    // (filter row, filter column, channel) of k0 once, then counted up element by element.  All
    // 16 fetches are issued before any is used (an element outside the image or past K fetches
    // the image's first code and is then dropped), so their latencies overlap.
    const int k32 = (int)k0, kend = (int)g.K;                          // K = kh kw Cin fits an int
    int tap = k32 / g.Cin, c = k32 - tap * g.Cin;
    int fr = tap / g.kw, fs = tap - fr * g.kw;
    uint32_t code[UNIT];
#pragma unroll
    for (int e = 0; e < UNIT; ++e) {
        const int hi = r.hi0 + fr, wi = r.wi0 + fs;
        const bool in = k32 + e < kend && (unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.Wd;
        const uint32_t v = fetch_code<BITS>(r.base + (in ? ((int64_t)hi * g.Wd + wi) * pix_bytes : 0), in ? c : 0);
        code[e] = in ? v : 0u;
        if (++c == g.Cin) {
            c = 0;
            if (++fs == g.kw) { fs = 0; ++fr; }
        }
    }
#pragma unroll
    for (int e = 0; e < UNIT; ++e) unit_set_code<BITS>(u, e, code[e]);
    return u;
}

template <int BITS, bool VECW>
__device__ __forceinline__ Unit<BITS> load_unit_W(const GemmArgs &g, const uint8_t *row, bool valid, int64_t k0)
{
    Unit<BITS> u;
#pragma unroll
    for (int i = 0; i < BITS / 2; ++i) u.w[i] = 0;
    if (!valid || k0 >= g.K) return u;
    if (VECW) return load_unit_vec<BITS>(row + k0 * BITS / 8);
    return load_unit_elems<BITS>(row, k0, g.K);
}

template <int BA, int BW, bool CONV, int MODE, bool WB>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(const GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) _Float16 As[BM * LDK];
    __shared__ __attribute__((aligned(16))) _Float16 Ws[BN * LDK];
    __shared__ uint32_t lutA[lut_entries<BA>()];
    __shared__ uint32_t lutW[lut_entries<BW>()];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t tiles_n = (g.N + BN - 1) / BN;
    const int64_t tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
    const int64_t m0 = tile_m * BM, n0 = tile_n * BN;

    build_lut<BA>(lutA, g.a_signed, tid);
    build_lut<BW>(lutW, g.w_signed, tid);

    // Each thread stages two units of A and two of W per K step: unit id -> (row, quarter of BK).
    constexpr int UPT = BM * (BK / UNIT) / GEMM_THREADS;   // = 2
    RowA ra[UPT];
    const uint8_t *rw[UPT];
    bool vw[UPT];
    int urow[UPT], ukq[UPT];
    const int64_t a_row_bytes = g.K * BA / 8, w_row_bytes = g.K * BW / 8;
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
        const int u = tid + i * GEMM_THREADS;
        urow[i] = u >> 2;
        ukq[i] = u & 3;
        const int64_t m = m0 + urow[i], n = n0 + urow[i];
        ra[i].valid = m < g.M;
        if (CONV) {
            const int64_t mm = ra[i].valid ? m : 0;
            const int64_t b = mm / ((int64_t)g.Ho * g.Wo);
            const int rem = (int)(mm - b * g.Ho * g.Wo);
            const int ho = rem / g.Wo, wo = rem - ho * g.Wo;
            ra[i].base = g.A + b * g.H * g.Wd * (int64_t)g.pix_bytes;
            ra[i].img_off = (uint32_t)(b * g.H * g.Wd * (int64_t)g.pix_bytes);     // RUNS: the tensor is below 2 GiB (and pixels are dense)
            ra[i].hi0 = ho * g.stride - g.pad;
            ra[i].wi0 = wo * g.stride - g.pad;
        } else {
            ra[i].base = g.A + (ra[i].valid ? m : 0) * a_row_bytes;
            ra[i].hi0 = ra[i].wi0 = 0;
            ra[i].img_off = 0;
        }
        vw[i] = n < g.N;
        rw[i] = g.W + (vw[i] ? n : 0) * w_row_bytes;
    }

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // RUNS: filter row and unit inside it of each staged unit, counted up from K step to K step
    // (a K step is BK / UNIT = 4 units further); the descriptor spans whole words of the tensor.
    const int units_per_row = MODE == RUNS ? g.kw * g.Cin / UNIT : 1;
    int run_fr[UPT], run_ur[UPT];
    const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(g.A), 0, MODE == RUNS ? (int)g.a_bytes : 0, 0x00020000);   // RUNS: whole words (checked by the entry point)
    auto next_run = [&](int i, int step) {
        run_ur[i] += step;
        while (run_ur[i] >= units_per_row) { run_ur[i] -= units_per_row; ++run_fr[i]; }
    };
    auto fetch_A = [&](int i, int64_t k0) -> Unit<BA> {
        if (MODE == RUNS) {
            const Unit<BA> u = load_unit_A_run<BA>(g, rsrcA, ra[i], run_fr[i], run_ur[i], k0);
            next_run(i, BK / UNIT);
            return u;
        }
        return load_unit_A<BA, CONV, MODE>(g, ra[i], k0);
    };
#pragma unroll
    for (int i = 0; i < UPT; ++i) { run_fr[i] = 0; run_ur[i] = 0; next_run(i, ukq[i]); }

    Unit<BA> ua[UPT];
    Unit<BW> uw[UPT];
    const int64_t ktiles = (g.K + BK - 1) / BK;
    if (ktiles > 0) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            ua[i] = fetch_A(i, (int64_t)ukq[i] * UNIT);
            uw[i] = load_unit_W<BW, MODE != ELEMS>(g, rw[i], vw[i], (int64_t)ukq[i] * UNIT);
        }
    }
    __syncthreads();   // tables ready

    for (int64_t kt = 0; kt < ktiles; ++kt) {
        // decode the staged units into the LDS tiles
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            u32x4 lo, hi;
            decode_unit<BA>(ua[i], lutA, lo, hi);
            u32x4 *dst = reinterpret_cast<u32x4 *>(&As[urow[i] * LDK + ukq[i] * UNIT]);
            dst[0] = lo; dst[1] = hi;
            decode_unit<BW>(uw[i], lutW, lo, hi);
            dst = reinterpret_cast<u32x4 *>(&Ws[urow[i] * LDK + ukq[i] * UNIT]);
            dst[0] = lo; dst[1] = hi;
        }
        __syncthreads();
        // fetch the next K step while the matrix cores work on this one
        if (kt + 1 < ktiles) {
            const int64_t kb = (kt + 1) * BK;
#pragma unroll
            for (int i = 0; i < UPT; ++i) {
                ua[i] = fetch_A(i, kb + ukq[i] * UNIT);
                uw[i] = load_unit_W<BW, MODE != ELEMS>(g, rw[i], vw[i], kb + ukq[i] * UNIT);
            }
        }
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            f16x8 fa[2], fw[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                fa[i] = *reinterpret_cast<const f16x8 *>(&As[(wm * 64 + i * 32 + (lane & 31)) * LDK + kk * 16 + (lane >> 5) * 8]);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fw[j] = *reinterpret_cast<const f16x8 *>(&Ws[(wn * 64 + j * 32 + (lane & 31)) * LDK + kk * 16 + (lane >> 5) * 8]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fw[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // epilogue (shared with the tiled kernels): each wave stores its two 32-row strips of 64 columns
    epilogue_strip<2, WB>(g, acc[0], m0 + wm * 64, n0 + wn * 64);
    epilogue_strip<2, WB>(g, acc[1], m0 + wm * 64 + 32, n0 + wn * 64);
}

template <int BA, int BW>
static void launch_gemm(const GemmArgs &g, bool conv, int mode, hipStream_t st)
{
    const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
    const dim3 grid((unsigned)tiles), block(GEMM_THREADS);
    note_kernel(DYBIT_KERNEL_GENERAL);
    if (conv) {
        if (mode == RUNS) hipLaunchKernelGGL((gemm_kernel<BA, BW, true, RUNS, kWriteBack>), grid, block, 0, st, g);
        else if (mode == VEC) hipLaunchKernelGGL((gemm_kernel<BA, BW, true, VEC, kWriteBack>), grid, block, 0, st, g);
        else hipLaunchKernelGGL((gemm_kernel<BA, BW, true, ELEMS, kWriteBack>), grid, block, 0, st, g);
    } else {
        if (mode == VEC) hipLaunchKernelGGL((gemm_kernel<BA, BW, false, VEC, kWriteBack>), grid, block, 0, st, g);
        else hipLaunchKernelGGL((gemm_kernel<BA, BW, false, ELEMS, kWriteBack>), grid, block, 0, st, g);
    }
}

// The write-back build of this file is compiled once per activation width (DYBIT_GEN_A = 2, 4, 6, 8:
// a quarter of the kernels each, so that the translation units compile side by side); the plain
// build holds all sixteen pairs.
#ifndef DYBIT_GEN_A
#define DYBIT_GEN_A 0
#endif
#if DYBIT_GEN_A == 0
void DYBIT_WB_NAME(launch_gemm_general)(const GemmArgs &g, int ba, int bw, bool conv, int mode, hipStream_t st)
{
#define DYBIT_G(A_, W_) case (A_) * 16 + (W_): launch_gemm<A_, W_>(g, conv, mode, st); break
    switch (ba * 16 + bw) {
        DYBIT_G(2, 2); DYBIT_G(2, 4); DYBIT_G(2, 6); DYBIT_G(2, 8);
        DYBIT_G(4, 2); DYBIT_G(4, 4); DYBIT_G(4, 6); DYBIT_G(4, 8);
        DYBIT_G(6, 2); DYBIT_G(6, 4); DYBIT_G(6, 6); DYBIT_G(6, 8);
        DYBIT_G(8, 2); DYBIT_G(8, 4); DYBIT_G(8, 6); DYBIT_G(8, 8);
    }
#undef DYBIT_G
}
#else
#define DYBIT_GEN_NAME2(a) DYBIT_WB_NAME(launch_gemm_general_a##a)
#define DYBIT_GEN_NAME(a) DYBIT_GEN_NAME2(a)
void DYBIT_GEN_NAME(DYBIT_GEN_A)(const GemmArgs &g, int bw, bool conv, int mode, hipStream_t st)
{
    switch (bw) {
        case 2: launch_gemm<DYBIT_GEN_A, 2>(g, conv, mode, st); break;
        case 4: launch_gemm<DYBIT_GEN_A, 4>(g, conv, mode, st); break;
        case 6: launch_gemm<DYBIT_GEN_A, 6>(g, conv, mode, st); break;
        case 8: launch_gemm<DYBIT_GEN_A, 8>(g, conv, mode, st); break;
    }
}
#endif

}  // namespace dybit

#if !DYBIT_WB && DYBIT_GEN_A == 0   // the C entry points live in the plain build of this file
using namespace dybit;

namespace {

// What happens to the accumulators on the way out: every entry point fills one of these.
struct Epilogue {
    const float *bias = nullptr, *residual = nullptr;
    int32_t relu = 0;
    float *absmax = nullptr;
    bool has_codes = false;          // write-back as DyBit codes requested
    dybit_fmt q_fmt{0, 0};
    const float *q_scale = nullptr;
    uint8_t *q_out = nullptr;
    bool w_per_channel = false;      // w_scale holds one value per output column
    const uint8_t *res_codes = nullptr;   // the shortcut as packed DyBit codes (needs the write-back form: q_out)
    dybit_fmt res_fmt{0, 0};
    const float *res_scale = nullptr;
};

// Checks the epilogue against the output shape and fills the matching fields of g.
// fp32 output `C` may be NULL only when codes are written.
dybit_status set_epilogue(GemmArgs &g, const Epilogue &e, float *C, int64_t ldc)
{
    g.bias = e.bias; g.relu = e.relu; g.residual = e.residual;
    g.w_per_channel = e.w_per_channel ? 1 : 0;
    g.absmax_bits = reinterpret_cast<uint32_t *>(e.absmax);
    g.C = C; g.ldc = ldc;
    if (!e.has_codes) return C ? DYBIT_OK : DYBIT_ERR_NULL;
    if (!e.q_out && !C) return DYBIT_ERR_NULL;
    if (!e.q_out) return DYBIT_OK;                                       // fp32 only after all
    if (!e.q_scale) return DYBIT_ERR_NULL;
    g.q_out = e.q_out; g.q_scale = e.q_scale;
    g.q_bits = e.q_fmt.bits; g.q_signed = e.q_fmt.is_signed;
    g.q_row_bytes = g.N * e.q_fmt.bits / 8;
    g.async_error = async_error_word();
    if (e.res_codes) {
        g.res_codes = e.res_codes; g.res_scale = e.res_scale;
        g.res_bits = e.res_fmt.bits; g.res_signed = e.res_fmt.is_signed;
        g.res_row_bytes = g.N * e.res_fmt.bits / 8;
    }
    return g.async_error ? DYBIT_OK : DYBIT_ERR_HIP;
}

// Argument checks of the write-back that need no device: format, whole words per row, sizes.
dybit_status check_codes_out(const Epilogue &e, int64_t N, int64_t ldc)
{
    if (!e.has_codes) return DYBIT_OK;
    const dybit_status st = check_fmt(e.q_fmt);
    if (st != DYBIT_OK) return st;
    if (e.q_fmt.bits == 2) return DYBIT_ERR_UNSUPPORTED_BITS;            // the epilogue packs 4-, 6- and 8-bit codes
    if ((N * e.q_fmt.bits) % 32) return DYBIT_ERR_ALIGNMENT;
    if (ldc >= (1 << 23) || N >= (1 << 23)) return DYBIT_ERR_INVALID_ARG;
    if (e.q_out && (reinterpret_cast<uintptr_t>(e.q_out) & 3u)) return DYBIT_ERR_ALIGNMENT;
    if (e.res_codes) {                                                   // shortcut as codes: only with codes out, whole bytes per row
        const dybit_status sr = check_fmt(e.res_fmt);
        if (sr != DYBIT_OK) return sr;
        if (e.res_fmt.bits == 2) return DYBIT_ERR_UNSUPPORTED_BITS;
        if (e.residual || !e.q_out) return DYBIT_ERR_INVALID_ARG;
        if (!e.res_scale) return DYBIT_ERR_NULL;
        if ((N * e.res_fmt.bits) % 8) return DYBIT_ERR_ALIGNMENT;
    }
    return DYBIT_OK;
}

dybit_status gemm_impl(int64_t M, int64_t N, int64_t K,
                       const uint8_t *A_codes, dybit_fmt a_fmt, const float *a_scale,
                       const uint8_t *W_codes, dybit_fmt w_fmt, const float *w_scale,
                       const Epilogue &e, float *C, int64_t ldc, dybit_stream stream)
{
    clear_call_record();
    dybit_status st = check_fmt(a_fmt);
    if (st == DYBIT_OK) st = check_fmt(w_fmt);
    if (st != DYBIT_OK) return st;
    if (M < 0 || N < 0 || K < 0 || ldc < N || (e.relu != 0 && e.relu != 1)) return DYBIT_ERR_INVALID_ARG;
    if ((K * a_fmt.bits) % 8 || (K * w_fmt.bits) % 8) return DYBIT_ERR_ALIGNMENT;
    if ((st = check_codes_out(e, N, ldc)) != DYBIT_OK) return st;
    if (M == 0 || N == 0) return DYBIT_OK;
    if (!a_scale || !w_scale || (K && (!A_codes || !W_codes))) return DYBIT_ERR_NULL;
    GemmArgs g{};
    g.M = M; g.N = N; g.K = K;
    g.A = A_codes; g.W = W_codes;
    g.a_signed = a_fmt.is_signed; g.w_signed = w_fmt.is_signed;
    g.a_scale = a_scale; g.w_scale = w_scale;
    if ((st = set_epilogue(g, e, C, ldc)) != DYBIT_OK) return st;
    g.a_bytes = M * (K * a_fmt.bits / 8);
    g.w_bytes = N * (K * w_fmt.bits / 8);
    if (launch_gemm_tiled(g, a_fmt.bits, w_fmt.bits, false, (hipStream_t)stream)) return launch_status();
    const int mode = (K % UNIT == 0) && aligned16(A_codes) && aligned16(W_codes) ? 1 : 0;   // VEC : ELEMS
    (g.q_out ? launch_gemm_general_wb : launch_gemm_general)(g, a_fmt.bits, w_fmt.bits, false, mode, (hipStream_t)stream);
    return launch_status();
}

dybit_status conv2d_impl(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                         int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                         const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                         const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale,
                         const Epilogue &e, float *Y, dybit_stream stream,
                         int64_t ldy = 0, int64_t image_channels = 0, int64_t x_bytes_left = 0)
{
    // ldy / image_channels / x_bytes_left (grouped convolution): X_codes and Y point at one channel group of
    // tensors with image_channels input and ldy output channels per pixel; x_bytes_left bytes of the image
    // tensor remain from X_codes on.  0: dense tensors of Cin and Cout channels.
    clear_call_record();
    dybit_status st = check_fmt(x_fmt);
    if (st == DYBIT_OK) st = check_fmt(w_fmt);
    if (st != DYBIT_OK) return st;
    if (B < 0 || H < 1 || W < 1 || Cin < 1 || Cout < 0 || kh < 1 || kw < 1 || stride < 1 || pad < 0 ||
        (e.relu != 0 && e.relu != 1) || H > (1 << 24) || W > (1 << 24) || Cin > (1 << 24))
        return DYBIT_ERR_INVALID_ARG;
    if (H + 2 * (int64_t)pad < kh || W + 2 * (int64_t)pad < kw) return DYBIT_ERR_INVALID_ARG;
    if ((int64_t)kh * kw > (1 << 24) || (int64_t)kh * kw * Cin > 0x7fffffff) return DYBIT_ERR_INVALID_ARG;   // K fits an int
    if ((Cin * x_fmt.bits) % 8 || (Cin * w_fmt.bits) % 8) return DYBIT_ERR_ALIGNMENT;
    if (ldy == 0) ldy = Cout;
    if (image_channels == 0) image_channels = Cin;
    if ((st = check_codes_out(e, Cout, ldy)) != DYBIT_OK) return st;
    const int64_t Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
    if (B == 0 || Cout == 0) return DYBIT_OK;
    if (!x_scale || !w_scale || !X_codes || !Wt_codes) return DYBIT_ERR_NULL;
    GemmArgs g{};
    g.M = B * Ho * Wo; g.N = Cout; g.K = (int64_t)kh * kw * Cin;
    g.A = X_codes; g.W = Wt_codes;
    g.a_signed = x_fmt.is_signed; g.w_signed = w_fmt.is_signed;
    g.a_scale = x_scale; g.w_scale = w_scale;
    if ((st = set_epilogue(g, e, Y, ldy)) != DYBIT_OK) return st;
    g.H = (int)H; g.Wd = (int)W; g.Cin = (int)Cin; g.Ho = (int)Ho; g.Wo = (int)Wo;
    g.kh = kh; g.kw = kw; g.stride = stride; g.pad = pad;
    g.pix_bytes = (int)(image_channels * x_fmt.bits / 8);
    const bool dense = image_channels == Cin;
    g.a_bytes = dense ? B * H * W * (Cin * x_fmt.bits / 8) : x_bytes_left;
    g.w_bytes = Cout * (g.K * w_fmt.bits / 8);
    if (launch_gemm_tiled(g, x_fmt.bits, w_fmt.bits, true, (hipStream_t)stream)) return launch_status();
    // operand access of the general kernel: whole 16-channel vectors, runs of neighbouring taps
    // when there are few channels (the first layer of an image network), else code by code
    const bool aligned = aligned16(X_codes) && aligned16(Wt_codes);
    int mode = 0;
    if (aligned && Cin % UNIT == 0) mode = 1;
    else if (aligned && dense && UNIT % Cin == 0 && ((int64_t)kw * Cin) % UNIT == 0 && g.a_bytes < 0x7fffffff && g.a_bytes % 4 == 0) mode = 2;
    (g.q_out ? launch_gemm_general_wb : launch_gemm_general)(g, x_fmt.bits, w_fmt.bits, true, mode, (hipStream_t)stream);
    return launch_status();
}

}  // namespace

extern "C" dybit_status dybit_gemm(int64_t M, int64_t N, int64_t K,
                                   const uint8_t *A_codes, dybit_fmt a_fmt, const float *a_scale,
                                   const uint8_t *W_codes, dybit_fmt w_fmt, const float *w_scale,
                                   const float *bias, int32_t relu,
                                   float *C, int64_t ldc, dybit_stream stream)
{
    Epilogue e;
    e.bias = bias; e.relu = relu;
    return gemm_impl(M, N, K, A_codes, a_fmt, a_scale, W_codes, w_fmt, w_scale, e, C, ldc, stream);
}

extern "C" dybit_status dybit_gemm_ex(int64_t M, int64_t N, int64_t K,
                                      const uint8_t *A_codes, dybit_fmt a_fmt, const float *a_scale,
                                      const uint8_t *W_codes, dybit_fmt w_fmt, const float *w_scale,
                                      const float *bias, const float *residual, int32_t relu,
                                      float *C, int64_t ldc, float *c_absmax, dybit_stream stream)
{
    Epilogue e;
    e.bias = bias; e.residual = residual; e.relu = relu; e.absmax = c_absmax;
    return gemm_impl(M, N, K, A_codes, a_fmt, a_scale, W_codes, w_fmt, w_scale, e, C, ldc, stream);
}

extern "C" dybit_status dybit_gemm_wb(int64_t M, int64_t N, int64_t K,
                                      const uint8_t *A_codes, dybit_fmt a_fmt, const float *a_scale,
                                      const uint8_t *W_codes, dybit_fmt w_fmt, const float *w_scale,
                                      const float *bias, const float *residual, int32_t relu,
                                      float *C, int64_t ldc, float *c_absmax,
                                      dybit_fmt c_fmt, const float *c_scale, uint8_t *C_codes, dybit_stream stream)
{
    Epilogue e;
    e.bias = bias; e.residual = residual; e.relu = relu; e.absmax = c_absmax;
    e.has_codes = true; e.q_fmt = c_fmt; e.q_scale = c_scale; e.q_out = C_codes;
    return gemm_impl(M, N, K, A_codes, a_fmt, a_scale, W_codes, w_fmt, w_scale, e, C, ldc, stream);
}

extern "C" dybit_status dybit_conv2d(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                     int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                     const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                                     const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale,
                                     const float *bias, int32_t relu,
                                     float *Y, dybit_stream stream)
{
    Epilogue e;
    e.bias = bias; e.relu = relu;
    return conv2d_impl(B, H, W, Cin, Cout, kh, kw, stride, pad, X_codes, x_fmt, x_scale, Wt_codes, w_fmt, w_scale, e, Y, stream);
}

extern "C" dybit_status dybit_conv2d_ex(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                        int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                        const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                                        const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale,
                                        const float *bias, const float *residual, int32_t relu,
                                        float *Y, float *y_absmax, dybit_stream stream)
{
    Epilogue e;
    e.bias = bias; e.residual = residual; e.relu = relu; e.absmax = y_absmax;
    return conv2d_impl(B, H, W, Cin, Cout, kh, kw, stride, pad, X_codes, x_fmt, x_scale, Wt_codes, w_fmt, w_scale, e, Y, stream);
}

extern "C" dybit_status dybit_conv2d_wb(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                        int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                        const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                                        const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale,
                                        const float *bias, const float *residual, int32_t relu,
                                        float *Y, float *y_absmax,
                                        dybit_fmt y_fmt, const float *y_scale, uint8_t *Y_codes, dybit_stream stream)
{
    Epilogue e;
    e.bias = bias; e.residual = residual; e.relu = relu; e.absmax = y_absmax;
    e.has_codes = true; e.q_fmt = y_fmt; e.q_scale = y_scale; e.q_out = Y_codes;
    return conv2d_impl(B, H, W, Cin, Cout, kh, kw, stride, pad, X_codes, x_fmt, x_scale, Wt_codes, w_fmt, w_scale, e, Y, stream);
}

extern "C" dybit_status dybit_gemm_wb_rc(int64_t M, int64_t N, int64_t K,
                                         const uint8_t *A_codes, dybit_fmt a_fmt, const float *a_scale,
                                         const uint8_t *W_codes, dybit_fmt w_fmt, const float *w_scale,
                                         const float *bias, const uint8_t *R_codes, dybit_fmt r_fmt, const float *r_scale,
                                         int32_t relu, float *C, int64_t ldc, float *c_absmax,
                                         dybit_fmt c_fmt, const float *c_scale, uint8_t *C_codes, dybit_stream stream)
{
    Epilogue e;
    e.bias = bias; e.relu = relu; e.absmax = c_absmax;
    e.res_codes = R_codes; e.res_fmt = r_fmt; e.res_scale = r_scale;
    e.has_codes = true; e.q_fmt = c_fmt; e.q_scale = c_scale; e.q_out = C_codes;
    if (!R_codes || !C_codes) return DYBIT_ERR_NULL;
    return gemm_impl(M, N, K, A_codes, a_fmt, a_scale, W_codes, w_fmt, w_scale, e, C, ldc, stream);
}

extern "C" dybit_status dybit_conv2d_wb_rc(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                           int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                           const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                                           const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale,
                                           const float *bias, const uint8_t *R_codes, dybit_fmt r_fmt, const float *r_scale,
                                           int32_t relu, float *Y, float *y_absmax,
                                           dybit_fmt y_fmt, const float *y_scale, uint8_t *Y_codes, dybit_stream stream)
{
    Epilogue e;
    e.bias = bias; e.relu = relu; e.absmax = y_absmax;
    e.res_codes = R_codes; e.res_fmt = r_fmt; e.res_scale = r_scale;
    e.has_codes = true; e.q_fmt = y_fmt; e.q_scale = y_scale; e.q_out = Y_codes;
    if (!R_codes || !Y_codes) return DYBIT_ERR_NULL;
    return conv2d_impl(B, H, W, Cin, Cout, kh, kw, stride, pad, X_codes, x_fmt, x_scale, Wt_codes, w_fmt, w_scale, e, Y, stream);
}

extern "C" dybit_status dybit_gemm_pc(int64_t M, int64_t N, int64_t K,
                                      const uint8_t *A_codes, dybit_fmt a_fmt, const float *a_scale,
                                      const uint8_t *W_codes, dybit_fmt w_fmt, const float *w_scales,
                                      const float *bias, const float *residual, int32_t relu,
                                      float *C, int64_t ldc, float *c_absmax,
                                      dybit_fmt c_fmt, const float *c_scale, uint8_t *C_codes, dybit_stream stream)
{
    Epilogue e;
    e.bias = bias; e.residual = residual; e.relu = relu; e.absmax = c_absmax; e.w_per_channel = true;
    e.has_codes = C_codes != nullptr; e.q_fmt = c_fmt; e.q_scale = c_scale; e.q_out = C_codes;
    return gemm_impl(M, N, K, A_codes, a_fmt, a_scale, W_codes, w_fmt, w_scales, e, C, ldc, stream);
}

extern "C" dybit_status dybit_conv2d_pc(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                        int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                        const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                                        const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scales,
                                        const float *bias, const float *residual, int32_t relu,
                                        float *Y, float *y_absmax,
                                        dybit_fmt y_fmt, const float *y_scale, uint8_t *Y_codes, dybit_stream stream)
{
    Epilogue e;
    e.bias = bias; e.residual = residual; e.relu = relu; e.absmax = y_absmax; e.w_per_channel = true;
    e.has_codes = Y_codes != nullptr; e.q_fmt = y_fmt; e.q_scale = y_scale; e.q_out = Y_codes;
    return conv2d_impl(B, H, W, Cin, Cout, kh, kw, stride, pad, X_codes, x_fmt, x_scale, Wt_codes, w_fmt, w_scales, e, Y, stream);
}
extern "C" dybit_status dybit_group_conv2d(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                           int32_t kh, int32_t kw, int32_t stride, int32_t pad, int32_t groups,
                                           const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                                           const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale, int32_t w_per_channel,
                                           const float *bias, const float *residual, int32_t relu,
                                           float *Y, float *y_absmax, dybit_stream stream)
{
    dybit_status st = check_fmt(x_fmt);
    if (st == DYBIT_OK) st = check_fmt(w_fmt);
    if (st != DYBIT_OK) return st;
    if (groups < 1 || Cin < 1 || Cout < 0 || Cin % groups || Cout % groups || (w_per_channel != 0 && w_per_channel != 1))
        return DYBIT_ERR_INVALID_ARG;
    const int64_t Cg = Cin / groups, Cog = Cout / groups;
    // a group's channels start on a byte of every pixel and of every filter
    if ((Cg * x_fmt.bits) % 8 || (Cg * w_fmt.bits) % 8 || (Cin * x_fmt.bits) % 8) return DYBIT_ERR_ALIGNMENT;
    if (B < 0 || H < 1 || W < 1 || kh < 1 || kw < 1) return DYBIT_ERR_INVALID_ARG;
    if (B == 0 || Cout == 0) return DYBIT_OK;
    if (!X_codes || !Wt_codes || !Y || !w_scale) return DYBIT_ERR_NULL;
    const int64_t x_bytes = B * H * W * (Cin * x_fmt.bits / 8);
    const int64_t group_x = Cg * x_fmt.bits / 8, group_w = Cog * ((int64_t)kh * kw * Cg * w_fmt.bits / 8);
    Epilogue e;
    e.relu = relu; e.absmax = y_absmax; e.w_per_channel = w_per_channel != 0;
    for (int64_t gi = 0; gi < groups; ++gi) {
        e.bias = bias ? bias + gi * Cog : nullptr;
        e.residual = residual ? residual + gi * Cog : nullptr;
        st = conv2d_impl(B, H, W, Cg, Cog, kh, kw, stride, pad, X_codes + gi * group_x, x_fmt, x_scale,
                         Wt_codes + gi * group_w, w_fmt, w_per_channel ? w_scale + gi * Cog : w_scale, e, Y + gi * Cog, stream,
                         Cout, Cin, x_bytes - gi * group_x);
        if (st != DYBIT_OK) return st;
    }
    return DYBIT_OK;
}
#endif   // plain build
