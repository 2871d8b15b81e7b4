// Large-tile DyBit matrix product for gfx950: 256 x 256 tile of C per workgroup, eight waves (two
// per SIMD); wave w owns rows 32 w .. 32 w + 31 of the tile and all 256 columns, i.e. 8 accumulator
// blocks of 32 x 32 in 128 AGPRs.  K step TK = 128 (K, for a convolution Cin, a multiple of 128) or 64.
//
// Why this shape.  Measured on this chip, a wave issues about one instruction per five cycles
// and every MFMA occupies the vector-ALU issue port for about twelve of its 32 cycles, so the
// decode arithmetic (the bulk of the instructions) must be spread over two waves per SIMD and
// nothing else may compete for issue slots.  LDS stores are the slow LDS operation (about 36
// cycles per 128-bit store per wave), LDS loads are not.  Hence:
//   * the activation operand A never touches LDS: every lane fetches the TK / 2 codes of its own
//     row that its MFMA fragments need (consecutive 128-bit buffer loads, two K steps ahead), decodes
//     them in registers and feeds the MFMA directly.  With one 32-row block per wave no A code is
//     decoded twice.  With TK = 128 the two lanes of a row together fetch 128 bytes of 8-bit codes,
//     one whole cache line per row and step, and there is one workgroup barrier per 128 k.
//   * the weight operand W is decoded once per workgroup (each thread TK / 2 codes per K step),
//     stored to a double-buffered LDS tile with one 128-bit store per 8 codes and read back by
//     all eight waves as MFMA fragments (`ds_read_b128`, rows padded by 16 B: no bank conflicts,
//     immediate offsets only) through a ring of four registers.
//   * decode is arithmetic / byte-permute work in the vector ALU, no table look-ups.
// A lane of k-group g (lane / 32) owns k = g TK/2 .. g TK/2 + TK/2 - 1 of every K step; MFMA block kk
// of a step contracts k = g TK/2 + 8 kk .. + 7.  The order of k inside an MFMA does not matter as
// long as both operands agree, so both codecs emit each group of eight k values in the order
// (k0,k2,k1,k3,k4,k6,k5,k7): that is the order their packed arithmetic produces for free.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <type_traits>

#include "dybit_codec.h"
#include "gemm_args.h"
#include "tile_common.h"
#include "tile_epilogue.h"

#ifndef DYBIT_FAST_W
#error "compile with -DDYBIT_FAST_W=<weight format id> (0: 4-bit signed, 2: 8-bit signed, 4: 6-bit signed, 6: 2-bit signed)"
#endif
#ifndef DYBIT_FAST_VALU_PER_MFMA
#define DYBIT_FAST_VALU_PER_MFMA 4     // vector-ALU instructions the scheduler places behind each MFMA
#endif

namespace dybit {
namespace fast {

constexpr int TM = 256, TN = 256;
template <int TK> struct Geom {
    static constexpr int KK = TK / 16;                         // MFMA k blocks per K step
    static constexpr int ROW_BYTES = TK * 2 + 16;              // one LDS row of W: TK halves plus 16 B of padding
    static constexpr int STAGE_BYTES = TN * ROW_BYTES;         // 36 KiB (TK = 64) or 68 KiB (TK = 128) per stage
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
};

// ---------------------------------------------------------------------------
// Kernel
// ---------------------------------------------------------------------------
template <int FMT_A, int FMT_W, bool CONV, int TK, bool WB>
__global__ __launch_bounds__(512) void gemm_fast_kernel(const GemmArgs g, const int tiles_m, const int tiles_n)
{
    using CA = Codec<FMT_A>;
    using CW = Codec<FMT_W>;
    using G = Geom<TK>;
    constexpr int KK = G::KK, ROW_BYTES = G::ROW_BYTES, STAGE_BYTES = G::STAGE_BYTES;
    // A lane's TK / 2 codes of a K step are consecutive bytes, fetched as whole 128-bit registers: 6-bit
    // codes (24 bytes per 32 codes) and 2-bit codes (8 bytes) therefore need the 128-wide K step.
    static_assert((TK / 2 * CA::BITS) % 128 == 0 && (TK / 2 * CW::BITS) % 128 == 0, "2- and 6-bit operands need TK = 128");
    constexpr int RUN_A = CA::BITS / 4, RUN_W = CW::BITS / 4;      // 128-bit registers per run of 32 codes (4-, 8-bit codes)
    constexpr int NA = TK / 2 * CA::BITS / 128;                    // 128-bit loads per lane and K step (consecutive bytes)
    constexpr int NW = TK / 2 * CW::BITS / 128;                    // ... per thread for W
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = lane >> 5;                                        // k-group of the lane

    // ---- tile assignment: consecutive workgroup ids go to different XCDs (8 of them, 32 compute
    // units each).  XCD x takes a contiguous range of a tile order that walks column panels of
    // 8 tiles row by row, so the 32 tiles it has in flight form a compact 4 x 8 patch whose
    // A and W strips are shared inside its own L2.  No workgroup is launched without a tile.
    int tile_m, tile_n;
    if (!panel_order_tile(xcd_contiguous_index(), tiles_m, tiles_n, tile_m, tile_n)) return;   // uniform per workgroup
    const int64_t m0 = (int64_t)tile_m * TM, n0 = (int64_t)tile_n * TN;

    const __amdgpu_buffer_rsrc_t rsrcA = code_descriptor(g.A, g.a_bytes), rsrcW = code_descriptor(g.W, g.w_bytes);

    // ---- A: the lane's own row, its k-group's half of the K step
    const int a_row_bytes = (int)(g.K * CA::BITS / 8), w_row_bytes = (int)(g.K * CW::BITS / 8);
    const int pix_bytes = CONV ? g.pix_bytes : 0;
    u32 offA;
    int hi0 = 0, wi0 = 0;
    const int64_t m_lane = m0 + wave * 32 + (lane & 31);
    const bool okA = m_lane < g.M;
    if (CONV) {
        const PixelOrigin o = pixel_origin(g, okA ? m_lane : 0);
        hi0 = o.hi0;
        wi0 = o.wi0;
        offA = (u32)(o.first_pixel * pix_bytes + kg * 16 * NA);
    } else {
        offA = okA ? (u32)(m_lane * a_row_bytes + kg * 16 * NA) : kOob;   // rows past M stay out of range as k advances
    }
    // ---- W staging: thread t decodes row t / 2, k-half t % 2
    const int wrow = tid >> 1, wh0 = tid & 1;
    const int64_t nrow = n0 + wrow;
    const u32 offW = nrow < g.N ? (u32)(nrow * w_row_bytes + wh0 * 16 * NW) : kOob;
    const u32 wrW = (u32)wrow * ROW_BYTES + (u32)wh0 * TK;                       // chunk KK h + q
    const u32 rdW = (u32)(lane & 31) * ROW_BYTES + (u32)kg * TK;                 // chunk KK g + kk, block j adds 32 rows

    // Tiles at or past ktiles (the prefetch of the last steps, and the padding step when the
    // number of K steps is odd) are fetched from an out-of-range offset: they read zeros.
    const int64_t ktiles = g.K / TK;
    // K steps are loaded in order, so for a convolution the filter row, filter column and first
    // channel of the next step are counted up instead of being divided out of k every time.
    TapCounter tap;
    auto load_A = [&](int64_t kt, u32x4 *raw) {
        u32 off;
        if (CONV) {
            const bool in = okA && tap.inside(g, hi0, wi0);
            off = (in && kt < ktiles) ? offA + (u32)tap.byte_offset(g, pix_bytes, CA::BITS) : kOob;   // padding reads code 0
            tap.advance(TK, g);
        } else {
            off = kt < ktiles ? offA + (u32)(kt * TK * CA::BITS / 8) : kOob;
        }
#pragma unroll
        for (int p = 0; p < NA; ++p) raw[p] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, off + p * 16, 0, 0);
    };
    auto load_W = [&](int64_t kt, u32x4 *raw) {
        const u32 off = kt < ktiles ? offW + (u32)(kt * TK * CW::BITS / 8) : kOob;
#pragma unroll
        for (int p = 0; p < NW; ++p) raw[p] = __builtin_amdgcn_raw_buffer_load_b128(rsrcW, off + p * 16, 0, 0);
    };
    // q: group of eight codes among the TK / 2 of the lane (run q / 4, group q % 4 of that run)
    auto decode_A = [&](const u32x4 *raw, int q) -> f16x8 {
        u32 d[4];
        if constexpr (CA::BITS == 6 || CA::BITS == 2) decode_eight<FMT_A>(raw, q, d);
        else decode_eight<FMT_A>(raw + (q >> 2) * RUN_A, q & 3, d);
        return __builtin_bit_cast(f16x8, u32x4{d[0], d[1], d[2], d[3]});
    };
    auto stage_W = [&](const u32x4 *raw, int q, char *tile) {
        u32 d[4];
        if constexpr (CW::BITS == 6 || CW::BITS == 2) decode_eight<FMT_W>(raw, q, d);
        else decode_eight<FMT_W>(raw + (q >> 2) * RUN_W, q & 3, d);
        *reinterpret_cast<u32x4 *>(tile + wrW + q * 16) = u32x4{d[0], d[1], d[2], d[3]};
    };
    auto read_W = [&](const char *tile, int kk, int j) -> f16x8 {
        return *reinterpret_cast<const f16x8 *>(tile + rdW + kk * 16 + j * 32 * ROW_BYTES);
    };

    f32x16 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;

    u32x4 rawA[2][NA], rawW[2][NW];
    f16x8 fw[4], fa;

    // ---- prologue: W tile 0 decoded into stage 0, A/W tile 1 in flight, first fragments in registers
    load_A(0, rawA[0]);
    load_W(0, rawW[0]);
    load_A(1, rawA[1]);
    load_W(1, rawW[1]);
#pragma unroll
    for (int q = 0; q < KK; ++q) stage_W(rawW[0], q, lds);
    fa = decode_A(rawA[0], 0);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) fw[j] = read_W(lds, 0, j);

    // One K step over LDS stage s: KK k blocks of 8 MFMAs.  The W fragments go through a ring of four
    // registers: as soon as the MFMA that uses one has issued, it is refilled with the fragment four
    // MFMAs ahead (column blocks 4..7 of this k block, then blocks 0..3 of the next).
    // The next W tile is decoded into the other stage during blocks 0..KK-2; the workgroup barrier
    // sits before the last block and the first fragments of the next tile are requested right after
    // it, so their LDS latency hides behind the MFMAs of that block.  The A fragment of block kk + 1
    // is decoded during block kk; the A codes of tile kt + 2 are fetched once tile kt's have
    // been consumed.  Every step is the same straight-line code (no tail variants: the
    // accumulators stay in place), so the last steps decode and prefetch tiles of zeros.
    auto step = [&](int64_t kt, auto stage_tag) {
        constexpr int s = decltype(stage_tag)::value;
        const char *cur = lds + s * STAGE_BYTES;
        char *nxt = lds + (s ^ 1) * STAGE_BYTES;
        load_W(kt + 2, rawW[s]);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            if (kk == KK - 1) __syncthreads();
            const f16x8 fa_cur = fa;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa_cur, fw[j & 3], acc[j], 0, 0, 0);
                if (j < 4) fw[j & 3] = read_W(cur, kk, j + 4);
                else fw[j & 3] = kk < KK - 1 ? read_W(cur, kk + 1, j - 4) : read_W(nxt, 0, j - 4);
            }
            fa = kk < KK - 1 ? decode_A(rawA[s], kk + 1) : decode_A(rawA[s ^ 1], 0);
            if (kk == 0) { stage_W(rawW[s ^ 1], 0, nxt); stage_W(rawW[s ^ 1], 1, nxt); }
            else if (kk < KK - 1) stage_W(rawW[s ^ 1], kk + 1, nxt);
            if (kk == KK - 2) load_A(kt + 2, rawA[s]);              // tile kt's codes are fully decoded by now
            // Issue order inside the block: an MFMA, the fragment refill behind it, a share of
            // the decode arithmetic.
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                 // DS read
                __builtin_amdgcn_sched_group_barrier(0x002, DYBIT_FAST_VALU_PER_MFMA, 0);   // VALU
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // an odd number of K steps is padded with one step of zeros
    for (int64_t kt = 0; kt < ktiles; kt += 2) {
        step(kt, std::integral_constant<int, 0>{});
        step(kt + 1, std::integral_constant<int, 1>{});
    }

    // ---- epilogue: C = acc * (sA sW) (+ bias) (ReLU), running maximum
    epilogue_strip<8, WB, true, CA::ACC_EXP + CW::ACC_EXP>(g, acc, m0 + wave * 32, n0);
}

template <int FA, int FW, bool CONV, int TK>
static void launch_tk(const GemmArgs &g, hipStream_t st)
{
    const int tiles_m = (int)((g.M + TM - 1) / TM), tiles_n = (int)((g.N + TN - 1) / TN);
    const dim3 grid((unsigned)((tiles_m * tiles_n + 7) / 8 * 8)), block(512);
    auto k = gemm_fast_kernel<FA, FW, CONV, TK, kWriteBack>;
    note_kernel(DYBIT_KERNEL_F16_256);
    note_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, Geom<TK>::LDS_BYTES));
    hipLaunchKernelGGL(k, grid, block, Geom<TK>::LDS_BYTES, st, g, tiles_m, tiles_n);
}

// K steps of 128 where a step never straddles a row end or a filter tap, else of 64 (not with a 2- or 6-bit
// operand, whose runs of 32 codes are not whole 128-bit registers: false, the caller takes another kernel).
template <int FA, int FW>
static bool launch(const GemmArgs &g, bool conv, hipStream_t st)
{
    constexpr bool six = Codec<FA>::BITS == 6 || Codec<FW>::BITS == 6 || Codec<FA>::BITS == 2 || Codec<FW>::BITS == 2;
    const bool wide = (conv ? g.Cin : g.K) % 128 == 0;
    if (six && !wide) return false;
    if (conv) {
        if (wide) launch_tk<FA, FW, true, 128>(g, st);
        else if constexpr (!six) launch_tk<FA, FW, true, 64>(g, st);
    } else {
        if (wide) launch_tk<FA, FW, false, 128>(g, st);
        else if constexpr (!six) launch_tk<FA, FW, false, 64>(g, st);
    }
    return true;
}

}  // namespace fast

// One translation unit per weight format (compile time); the entry point's name carries it.
#define DYBIT_FAST_NAME2(w) DYBIT_WB_NAME(launch_gemm_fast_w##w)
#define DYBIT_FAST_NAME(w) DYBIT_FAST_NAME2(w)
bool DYBIT_FAST_NAME(DYBIT_FAST_W)(const GemmArgs &g, int a_bits, bool conv, hipStream_t st)
{
    using namespace fast;
    const int fa = (a_bits == 8 ? F8S : a_bits == 6 ? F6S : a_bits == 2 ? F2S : F4S) + (g.a_signed ? 0 : 1);
    switch (fa) {
        case F2S: return fast::launch<F2S, DYBIT_FAST_W>(g, conv, st);
        case F2U: return fast::launch<F2U, DYBIT_FAST_W>(g, conv, st);
        case F4S: return fast::launch<F4S, DYBIT_FAST_W>(g, conv, st);
        case F4U: return fast::launch<F4U, DYBIT_FAST_W>(g, conv, st);
        case F6S: return fast::launch<F6S, DYBIT_FAST_W>(g, conv, st);
        case F6U: return fast::launch<F6U, DYBIT_FAST_W>(g, conv, st);
        case F8S: return fast::launch<F8S, DYBIT_FAST_W>(g, conv, st);
        case F8U: return fast::launch<F8U, DYBIT_FAST_W>(g, conv, st);
        default: return false;
    }
}

}  // namespace dybit
