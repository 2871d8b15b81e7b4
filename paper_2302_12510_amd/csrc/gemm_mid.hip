// Mid-size-tile DyBit matrix product for gfx950: 128 x 128 tile of C per workgroup, for shapes
// that do not have enough 256 x 256 tiles to fill the 256 compute units (the convolution
// layers of a network, a GEMM with a narrow N).  Two variants, by the number KG of k-groups:
//
// KG = 1: four waves, wave w owns rows 32 w .. 32 w + 31 and all 128 columns, K step 64.
//   Three workgroups fit on a compute unit (three waves per SIMD), so that one workgroup's
//   decode arithmetic, its prologue and its epilogue overlap the MFMAs of the others.  Used when
//   there are more tiles than compute units.
// KG = 2: eight waves, two per SIMD inside one workgroup, for problems with at most one tile per
//   compute unit.  With a 128 x 128 tile there are only four 32-row strips, so the eight waves
//   are four row strips x two k-groups: a K step is 128 wide, k-group g contracts
//   k = 64 g .. 64 g + 63 of it, and the two partial accumulators of a row strip are added
//   through LDS once, after the K loop.
// Per wave and K step: four MFMA k blocks of 16 -> 16 MFMAs into 4 accumulator blocks (64
// registers).
//
// Operand paths are those of the large-tile kernel: the activation operand A is fetched by the
// lane that needs it (its row, its 32 consecutive k) and decoded straight into MFMA fragments;
// the weight operand W is decoded once per workgroup (each thread 32 codes of one row) into a
// double-buffered LDS tile (rows padded by 16 B) and read back as fragments by every wave.
// Codes past K, rows past M / N and filter taps outside the image are fetched from an
// out-of-range buffer offset and read as code 0 = 0.0, so K only has to be a multiple of 64.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <type_traits>

#include "dybit_codec.h"
#include "gemm_args.h"
#include "tile_common.h"
#include "tile_epilogue.h"

#ifndef DYBIT_MID_W
#error "compile with -DDYBIT_MID_W=<weight format id> (0: 4-bit signed, 2: 8-bit signed)"
#endif

namespace dybit {
namespace mid {

using namespace fast;

constexpr int TM = 128, TN = 128;

template <int KG> struct Geom {
    static constexpr int TK = 64 * KG;
    static constexpr int ROW_BYTES = TK * 2 + 16;         // one LDS row of W: TK halves plus 16 B of padding
    static constexpr int STAGE_BYTES = TN * ROW_BYTES;    // 18 KiB (KG = 1) or 34 KiB (KG = 2) per stage
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;     // KG = 2: also holds the 64 KiB of partial sums at the end
};
static_assert(Geom<2>::LDS_BYTES >= 4 * 4 * 16 * 64 * 4, "reduction buffer must fit in the stages");

// CONV: 0 matrix product; 1 convolution whose 64-code k groups lie inside one filter tap (Cin a multiple
// of 64); 2 (ROWS) convolution with few channels where one filter row is exactly one 32-code run
// (kw * Cin = 32, e.g. 8 taps of 4 channels: the first layer of an image network with its weights
// padded by zero taps): a lane's run is filter row 2 * step + kq of its output pixel, contiguous in
// the image from any byte on.  It is fetched as aligned words (one more than the run holds; a word
// before or past the tensor reads 0) and, when it is decoded, shifted into place and the taps left or
// right of the image are masked to code 0.
constexpr int ROWS = 2;

template <int FMT_A, int FMT_W, int CONV, int KG, bool WB>
__global__ __launch_bounds__(256 * KG, (KG == 1) ? 3 : 2) void gemm_mid_kernel(const GemmArgs g, const int tiles_m, const int tiles_n)
{
    using CA = Codec<FMT_A>;
    using CW = Codec<FMT_W>;
    constexpr int TK = Geom<KG>::TK, ROW_BYTES = Geom<KG>::ROW_BYTES, STAGE_BYTES = Geom<KG>::STAGE_BYTES;
    constexpr int WORDS_A = CA::BITS;                               // 32-bit words in a run of 32 codes
    constexpr int NA = CONV == ROWS ? (WORDS_A + 1 + 3) / 4 : (CA::BITS + 3) / 4;   // 128-bit registers per lane and K step
    constexpr int NW = (CW::BITS + 3) / 4;
    constexpr int RUN_A = 4 * CA::BITS, RUN_W = 4 * CW::BITS;       // bytes of a run of 32 codes
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave & 3, kgp = wave >> 2;                        // row strip and k-group of the wave
    const int kq = lane >> 5;                                        // which 32 k of the k-group's 64 the lane owns

    // ---- tile assignment: consecutive workgroup ids go to different XCDs; give each XCD a
    // contiguous range of tiles (all column tiles of a row strip together), so that the A rows
    // it streams are shared inside its own L2.
    int tile_m, tile_n;
    if (!row_order_tile(xcd_contiguous_index(), tiles_m, tiles_n, tile_m, tile_n)) return;   // uniform per workgroup
    const int64_t m0 = (int64_t)tile_m * TM, n0 = (int64_t)tile_n * TN;

    // ROWS reads aligned words; the dispatcher takes it only for tensors of a whole number of words, so
    // the descriptor ends exactly with the tensor and no word reaches past it
    const __amdgpu_buffer_rsrc_t rsrcA = code_descriptor(g.A, g.a_bytes), rsrcW = code_descriptor(g.W, g.w_bytes);

    // ---- A: the lane's own row, the 32 codes kq of its k-group's 64
    const int a_row_bytes = (int)(g.K * CA::BITS / 8), w_row_bytes = (int)(g.K * CW::BITS / 8);
    const int pix_bytes = CONV ? g.pix_bytes : 0;
    u32 offA;
    int hi0 = 0, wi0 = 0;
    bool okA;
    // ROWS: byte shift of the lane's runs inside their aligned words, and the bits of the run that
    // belong to taps inside the image (both the same for every filter row of the pixel)
    u32 row_shift = 0, row_keep[CONV == ROWS ? WORDS_A : 1];
    {
        const int64_t m = m0 + wr * 32 + (lane & 31);
        okA = m < g.M;
        if (CONV) {
            const PixelOrigin o = pixel_origin(g, okA ? m : 0);
            hi0 = o.hi0;
            wi0 = o.wi0;
            if (CONV == ROWS) {
                // first byte of filter row 0 of the pixel (negative left of the first pixel of the tensor)
                const int first = (int)(o.first_pixel * pix_bytes);
                row_shift = (u32)first & 3u;                     // Wd * pix_bytes may be odd: see load_A
                offA = (u32)first;
                const int taps = 32 / g.Cin, tap_bits = g.Cin * CA::BITS;
                const int t_lo = max(0, -wi0), t_hi = max(min(taps, g.Wd - wi0), t_lo);
#pragma unroll
                for (int i = 0; i < WORDS_A; ++i) {
                    const int lo = min(max(t_lo * tap_bits - 32 * i, 0), 32), up = min(max(t_hi * tap_bits - 32 * i, 0), 32);
                    row_keep[i] = (u32)((1ull << up) - 1ull) & ~(u32)((1ull << lo) - 1ull);
                }
            } else {
                offA = (u32)(o.first_pixel * pix_bytes + kq * RUN_A);
            }
        } else {
            offA = okA ? (u32)(m * a_row_bytes + kq * RUN_A) : kOob;
        }
    }
    // ---- W staging: a row of the K step is TK / 32 = 2 KG runs of 32 codes, one thread each
    const int wrow = tid / (2 * KG), wq = tid % (2 * KG);
    const int64_t nrow = n0 + wrow;
    const u32 offW = nrow < g.N ? (u32)(nrow * w_row_bytes + wq * RUN_W) : kOob;
    const u32 wrW = (u32)wrow * ROW_BYTES + (u32)wq * 64;
    const u32 rdW = (u32)(lane & 31) * ROW_BYTES + (u32)kgp * 128 + (u32)kq * 64;   // block kk adds 16 B, column block j adds 32 rows

    // K steps are loaded in order, so the position of the next one is counted up instead of being
    // divided out of k every time: first k of the wave's k-group, and for a convolution its filter
    // row, filter column and first channel (all uniform over the wave, hence the readfirstlane above).
    int64_t a_k0 = kgp * 64;
    TapCounter tap;
    if (CONV == 1) tap.advance(kgp * 64, g);
    auto load_A = [&](u32x4 *raw) {
        if constexpr (CONV == ROWS) {
            // filter row of this lane's run, its first byte, and the aligned words that hold it; the
            // byte shift travels with the words (last register) because rows may start at any byte
            const int fr = (int)(a_k0 >> 5) + kq;
            const int hi = hi0 + fr;
            const bool in = okA && a_k0 < g.K && (unsigned)hi < (unsigned)g.H;
            const int byte_off = (int)offA + fr * g.Wd * pix_bytes;
            const int shift = byte_off & 3, base = byte_off - shift;
            u32 w[NA * 4];
#pragma unroll
            for (int j = 0; j < NA * 4; ++j) w[j] = 0;
#pragma unroll
            for (int j = 0; j <= WORDS_A; ++j) {
                const int o = base + 4 * j;                      // no wrap-around in the hardware's offset addition:
                w[j] = __builtin_amdgcn_raw_buffer_load_b32(rsrcA, (in && o >= 0) ? (u32)o : kOob, 0, 0);   // say "outside" explicitly
            }
            w[NA * 4 - 1] = (u32)shift;
#pragma unroll
            for (int p = 0; p < NA; ++p) raw[p] = u32x4{w[4 * p], w[4 * p + 1], w[4 * p + 2], w[4 * p + 3]};
            a_k0 += TK;
            return;
        }
        u32 off;
        if (CONV) {
            const bool in = okA && a_k0 < g.K && tap.inside(g, hi0, wi0);
            off = in ? offA + (u32)tap.byte_offset(g, pix_bytes, CA::BITS) : kOob;   // padding reads code 0
        } else {
            off = a_k0 < g.K ? offA + (u32)(a_k0 * CA::BITS / 8) : kOob;
        }
        load_run<CA::BITS>(rsrcA, off, raw);
        a_k0 += TK;
        if (CONV == 1) tap.advance(TK, g);
    };
    auto load_W = [&](int64_t kt, u32x4 *raw) {
        const int64_t k0 = kt * TK + wq * 32;
        const u32 off = k0 < g.K ? offW + (u32)(kt * TK * CW::BITS / 8) : kOob;
        load_run<CW::BITS>(rsrcW, off, raw);
    };
    auto decode_A = [&](const u32x4 *raw, int q) -> f16x8 {
        u32 d[4];
        if constexpr (CONV == ROWS) {
            // shift the run into place and drop the taps outside the image (only the words group q
            // needs survive dead-code elimination: q is a constant where this is inlined)
            const u32 shift = raw[NA - 1].w;
            u32x4 t[2] = {u32x4{0u, 0u, 0u, 0u}, u32x4{0u, 0u, 0u, 0u}};
#pragma unroll
            for (int i = 0; i < WORDS_A; ++i)
                t[i >> 2][i & 3] = __builtin_amdgcn_alignbyte(raw[(i + 1) >> 2][(i + 1) & 3], raw[i >> 2][i & 3], shift) & row_keep[i];
            decode_eight<FMT_A>(t, q, d);
        } else {
            decode_eight<FMT_A>(raw, q, d);
        }
        return __builtin_bit_cast(f16x8, u32x4{d[0], d[1], d[2], d[3]});
    };
    auto stage_W = [&](const u32x4 *raw, int q, char *tile) {
        u32 d[4];
        decode_eight<FMT_W>(raw, q, d);
        *reinterpret_cast<u32x4 *>(tile + wrW + q * 16) = u32x4{d[0], d[1], d[2], d[3]};
    };
    auto read_W = [&](const char *tile, int kk, int j) -> f16x8 {
        return *reinterpret_cast<const f16x8 *>(tile + rdW + kk * 16 + j * 32 * ROW_BYTES);
    };

    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;

    // decode instructions to place behind each MFMA: the 6-bit decoders are about 1.5 times as long
    constexpr int VALU_PER_MFMA = 12 + (CA::BITS == 6 ? 6 : 0) + (CW::BITS == 6 ? 6 : 0);
    u32x4 rawA[2][NA], rawW[2][NW];
    f16x8 fw[4], fa;

    // ---- prologue: W tile 0 decoded into stage 0, A/W tile 1 in flight, first fragments in registers
    load_A(rawA[0]);
    load_W(0, rawW[0]);
    load_A(rawA[1]);
    load_W(1, rawW[1]);
#pragma unroll
    for (int q = 0; q < 4; ++q) stage_W(rawW[0], q, lds);
    fa = decode_A(rawA[0], 0);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) fw[j] = read_W(lds, 0, j);

    // One K step over LDS stage s: four k blocks of four MFMAs.  A W fragment register is refilled
    // with the next block's fragment right after the MFMA that used it; the next W tile is decoded
    // into the other stage during blocks 0..2; the workgroup barrier sits before block 3 and the
    // first fragments of the next tile are requested right after it.  The A fragment of block
    // kk + 1 is decoded during block kk.  Every step is the same straight-line code, so the last
    // steps decode and prefetch tiles of zeros.
    auto step = [&](int64_t kt, auto stage_tag) {
        constexpr int s = decltype(stage_tag)::value;
        const char *cur = lds + s * STAGE_BYTES;
        char *nxt = lds + (s ^ 1) * STAGE_BYTES;
        load_W(kt + 2, rawW[s]);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk == 3) __syncthreads();
            const f16x8 fa_cur = fa;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa_cur, fw[j], acc[j], 0, 0, 0);
                fw[j] = kk < 3 ? read_W(cur, kk + 1, j) : read_W(nxt, 0, j);
            }
            fa = kk < 3 ? decode_A(rawA[s], kk + 1) : decode_A(rawA[s ^ 1], 0);
            if (kk == 0) { stage_W(rawW[s ^ 1], 0, nxt); stage_W(rawW[s ^ 1], 1, nxt); }
            if (kk == 1) stage_W(rawW[s ^ 1], 2, nxt);
            if (kk == 2) stage_W(rawW[s ^ 1], 3, nxt);
            if (kk == 2) load_A(rawA[s]);                           // K step kt + 2; tile kt's codes are fully decoded by now
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                 // DS read
                __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER_MFMA, 0);     // VALU
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    const int64_t ktiles = (g.K + TK - 1) / TK;
    for (int64_t kt = 0; kt < ktiles; kt += 2) {                   // an odd number of K steps is padded with a step of zeros
        step(kt, std::integral_constant<int, 0>{});
        step(kt + 1, std::integral_constant<int, 1>{});
    }

    // ---- add the two k-groups' partial sums: k-group 1 hands its accumulators over through LDS
    if constexpr (KG == 2) {
        __syncthreads();                                            // every fragment read has completed
        float *red = reinterpret_cast<float *>(lds);
        if (kgp == 1) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) red[((wr * 4 + j) * 16 + v) * 64 + lane] = acc[j][v];
        }
        __syncthreads();
        if (kgp == 1) return;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][v] += red[((wr * 4 + j) * 16 + v) * 64 + lane];
    }

    // ---- epilogue: C = acc * (sA sW) (+ bias) (ReLU), running maximum
    epilogue_strip<4, WB, true, CA::ACC_EXP + CW::ACC_EXP>(g, acc, m0 + wr * 32, n0);
}

template <int FA, int FW, int CONV, int KG>
static void launch_one(const GemmArgs &g, hipStream_t st, int tiles_m, int tiles_n)
{
    const dim3 grid((unsigned)((tiles_m * tiles_n + 7) / 8 * 8), 1, 1), block(256 * KG);
    constexpr int lds_bytes = Geom<KG>::LDS_BYTES;
    auto k = gemm_mid_kernel<FA, FW, CONV, KG, kWriteBack>;
    note_kernel(CONV == ROWS ? DYBIT_KERNEL_F16_128_ROWS : KG == 1 ? DYBIT_KERNEL_F16_128_KG1 : DYBIT_KERNEL_F16_128_KG2);
    note_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
    hipLaunchKernelGGL(k, grid, block, lds_bytes, st, g, tiles_m, tiles_n);
}

template <int FA, int FW, int KG>
static void launch_kg(const GemmArgs &g, bool conv, hipStream_t st, int tiles_m, int tiles_n)
{
    if (conv) launch_one<FA, FW, 1, KG>(g, st, tiles_m, tiles_n);
    else launch_one<FA, FW, 0, KG>(g, st, tiles_m, tiles_n);
}

// More tiles than compute units: small workgroups, three per compute unit.  Otherwise one
// eight-wave workgroup per compute unit.  The "mid_kgroups" option overrides (tests).
template <int FA, int FW>
static void launch(const GemmArgs &g, bool conv, hipStream_t st)
{
    const int tiles_m = (int)((g.M + TM - 1) / TM), tiles_n = (int)((g.N + TN - 1) / TN);
    if (conv && g.Cin < 64) return launch_one<FA, FW, ROWS, 1>(g, st, tiles_m, tiles_n);   // kw * Cin = 32 (checked by the dispatcher)
    const int force = dispatch_options().mid_kgroups;
    const bool one = force ? force == 1 : (int64_t)tiles_m * tiles_n > 256;
    if (one) launch_kg<FA, FW, 1>(g, conv, st, tiles_m, tiles_n);
    else launch_kg<FA, FW, 2>(g, conv, st, tiles_m, tiles_n);
}

}  // namespace mid

// One translation unit per weight format (compile time); the entry point's name carries it.
#define DYBIT_MID_NAME2(w) DYBIT_WB_NAME(launch_gemm_mid_w##w)
#define DYBIT_MID_NAME(w) DYBIT_MID_NAME2(w)
bool DYBIT_MID_NAME(DYBIT_MID_W)(const GemmArgs &g, int a_bits, bool conv, hipStream_t st)
{
    using namespace fast;
    const int fa = (a_bits == 8 ? F8S : a_bits == 6 ? F6S : a_bits == 2 ? F2S : F4S) + (g.a_signed ? 0 : 1);
    switch (fa) {
        case F2S: mid::launch<F2S, DYBIT_MID_W>(g, conv, st); return true;
        case F2U: mid::launch<F2U, DYBIT_MID_W>(g, conv, st); return true;
        case F4S: mid::launch<F4S, DYBIT_MID_W>(g, conv, st); return true;
        case F4U: mid::launch<F4U, DYBIT_MID_W>(g, conv, st); return true;
        case F6S: mid::launch<F6S, DYBIT_MID_W>(g, conv, st); return true;
        case F6U: mid::launch<F6U, DYBIT_MID_W>(g, conv, st); return true;
        case F8S: mid::launch<F8S, DYBIT_MID_W>(g, conv, st); return true;
        case F8U: mid::launch<F8U, DYBIT_MID_W>(g, conv, st); return true;
        default: return false;
    }
}

}  // namespace dybit
