// DyBit matrix product for pairs of 4-bit and 2-bit formats on the fp8 matrix path of gfx950
// (`v_mfma_f32_32x32x64_f8f6f4` with both operands e4m3): every value of the 4-bit formats has at
// most 3 significant bits and lies in [1/8, 8], and the 2-bit formats hold 0, 1/2, 1, 2 or 0, +-1, so
// all are exact in e4m3; one instruction contracts 64 k in the time the fp16 instruction needs for
// 32, and the decoders emit bytes, not halves.
//
// Same organisation as the fp16 kernels (gemm_fast.hip, gemm_mid.hip): square tile of 32 NWM rows
// and columns; NWM x KG waves; wave (wr, g) owns rows 32 wr .. + 31, all columns (CB = NWM
// accumulator blocks) and, of every K step of 128 KG, the k-group k = 128 g .. 128 g + 127, which
// is two MFMA blocks of 64.  Lane (row, kq = lane / 32) of the A operand supplies k = 32 kq .. + 31
// of a block: 32 codes = one 128-bit (2-bit codes: 64-bit) load, decoded in registers straight into
// the 32-byte fragment.
// W is decoded once per workgroup (each thread 64 codes of one row) into a double-buffered LDS tile
// of bytes (rows padded by 16 B) and read back as 32-byte fragments through a ring of two fragment
// registers that is refilled right behind the MFMAs.  KG = 2 k-groups add their accumulators
// through LDS after the K loop.  Configurations:
//   NWM = 8, KG = 1   256 x 256 tile, 8 waves (two per SIMD)               many large tiles
//   NWM = 4, KG = 1   128 x 128 tile, 4 waves, three workgroups per CU     more tiles than CUs
//   NWM = 4, KG = 2   128 x 128 tile, 8 waves                              at most one tile per CU
//   NWM = 2, KG = 2   64 x 64 tile, 4 waves, four workgroups per CU        128 x 128 tiles for under half the CUs
// The order of the 32 k inside a lane's fragment is the one the 4-bit decoders produce (per eight
// consecutive codes: the four even ones, then the four odd ones); the 2-bit decoders emit the same
// order, and the instruction pairs byte i of an A lane with byte i of the B lane of the same
// k-quarter.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <type_traits>

#include "dybit_codec.h"
#include "dybit_codec8.h"
#include "gemm_args.h"
#include "tile_common.h"
#include "tile_epilogue.h"

namespace dybit {
namespace f8 {

using namespace fast;

template <int NWM, int KG> struct Geom {
    static constexpr int T = 32 * NWM;                    // tile rows = tile columns
    static constexpr int TK = 128 * KG;
    static constexpr int ROW_BYTES = TK + 16;             // one LDS row of W: TK bytes plus 16 B of padding
    static constexpr int STAGE_BYTES = T * ROW_BYTES;
    static constexpr int RED_BYTES = KG == 2 ? NWM * NWM * 16 * 64 * 4 : 0;   // partial sums of k-group 1
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES > RED_BYTES ? 2 * STAGE_BYTES : RED_BYTES;
    static constexpr int THREADS = 64 * NWM * KG;
};

template <int FMT_A, int FMT_W, bool CONV, int NWM, int KG, bool WB>
__global__ __launch_bounds__(64 * NWM * KG, NWM == 2 ? 4 : (NWM == 4 && KG == 1) ? 3 : 2)
void gemm_f8_kernel(const GemmArgs g, const int tiles_m, const int tiles_n)
{
    using G = Geom<NWM, KG>;
    constexpr int T = G::T, TK = G::TK, ROW_BYTES = G::ROW_BYTES, STAGE_BYTES = G::STAGE_BYTES;
    constexpr int CB = NWM;                                        // 32-column blocks per wave
    constexpr int NQ = 2 * CB;                                     // MFMAs per wave and K step
    constexpr int R = 2;                                           // W fragment registers (ring); more would spill
    constexpr int BA = bits_of<FMT_A>(), BW = bits_of<FMT_W>();    // code widths
    constexpr int A_LOAD = 4 * BA;                                 // bytes of a lane's 32 codes of A
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave % NWM, kgp = wave / NWM;                     // row strip and k-group of the wave
    const int kq = lane >> 5;                                        // which 32 k of a 64-wide block the lane owns

    // ---- tile assignment: XCD x (workgroup id mod 8) takes a contiguous range of a tile order that
    // walks column panels of up to 8 tiles row by row
    int tile_m, tile_n;
    if (!panel_order_tile(xcd_contiguous_index(), tiles_m, tiles_n, tile_m, tile_n)) return;   // uniform per workgroup
    const int64_t m0 = (int64_t)tile_m * T, n0 = (int64_t)tile_n * T;

    const __amdgpu_buffer_rsrc_t rsrcA = code_descriptor(g.A, g.a_bytes), rsrcW = code_descriptor(g.W, g.w_bytes);

    // ---- A: the lane's own row; per 64-wide block its 32 codes (16 bytes) at k-quarter kq
    const int a_row_bytes = (int)(g.K * BA / 8), w_row_bytes = (int)(g.K * BW / 8);
    const int pix_bytes = CONV ? g.pix_bytes : 0;
    u32 offA;
    int hi0 = 0, wi0 = 0;
    bool okA;
    {
        const int64_t m = m0 + wr * 32 + (lane & 31);
        okA = m < g.M;
        if (CONV) {
            const PixelOrigin o = pixel_origin(g, okA ? m : 0);
            hi0 = o.hi0;
            wi0 = o.wi0;
            offA = (u32)(o.first_pixel * pix_bytes + kq * A_LOAD);
        } else {
            offA = okA ? (u32)(m * a_row_bytes + kq * A_LOAD) : kOob;
        }
    }
    // ---- W staging: a row of the K step is 2 KG runs of 64 codes, one thread each
    const int wrow = tid / (2 * KG), wp = tid % (2 * KG);
    const int64_t nrow = n0 + wrow;
    const u32 offW = nrow < g.N ? (u32)(nrow * w_row_bytes + wp * (8 * BW)) : kOob;
    const u32 wrW = (u32)wrow * ROW_BYTES + (u32)wp * 64;
    const u32 rdW = (u32)(lane & 31) * ROW_BYTES + (u32)kgp * 128 + (u32)kq * 32;   // block b adds 64 B, column block j adds 32 rows

    // K steps are loaded in order: the first k of the wave's next block, and for a convolution its
    // filter row, filter column and first channel, are counted up (uniform over the wave).
    int64_t a_k0 = kgp * 128;
    TapCounter tap;
    if (CONV) tap.advance(kgp * 128, g);
    auto load_A_block = [&](u32x4 &raw, int advance) {                  // one 64-wide block, then step on by `advance`
        u32 off;
        if (CONV) {
            const bool in = okA && a_k0 < g.K && tap.inside(g, hi0, wi0);
            off = in ? offA + (u32)tap.byte_offset(g, pix_bytes, BA) : kOob;   // padding reads code 0
        } else {
            off = a_k0 < g.K ? offA + (u32)(a_k0 * BA / 8) : kOob;
        }
        if constexpr (BA == 2) {
            const u32x2 two = __builtin_amdgcn_raw_buffer_load_b64(rsrcA, off, 0, 0);
            raw = u32x4{two.x, two.y, 0u, 0u};
        } else {
            raw = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, off, 0, 0);
        }
        a_k0 += advance;
        if (CONV) tap.advance(advance, g);
    };
    auto load_A = [&](u32x4 *raw) {                                       // both blocks of the next K step
        load_A_block(raw[0], 64);
        load_A_block(raw[1], TK - 64);
    };
    auto load_W = [&](int64_t kt, u32x4 *raw) {
        const int64_t k0 = kt * TK + wp * 64;
        const u32 off = k0 < g.K ? offW + (u32)(kt * (TK * BW / 8)) : kOob;     // K is a multiple of 64
        raw[0] = __builtin_amdgcn_raw_buffer_load_b128(rsrcW, off, 0, 0);       // 4-bit: 32 codes; 2-bit: all 64
        if constexpr (BW == 4) raw[1] = __builtin_amdgcn_raw_buffer_load_b128(rsrcW, off + 16, 0, 0);
    };
    auto stage_W = [&](const u32x4 *raw, int h, char *tile) {              // half h of the thread's 64 codes -> 32 bytes
        const i32x8 f = BW == 4 ? decode_fragment<FMT_W>(raw[h]) : decode_fragment<FMT_W>(raw[0], h);
        *reinterpret_cast<u32x4 *>(tile + wrW + h * 32) = u32x4{(u32)f[0], (u32)f[1], (u32)f[2], (u32)f[3]};
        *reinterpret_cast<u32x4 *>(tile + wrW + h * 32 + 16) = u32x4{(u32)f[4], (u32)f[5], (u32)f[6], (u32)f[7]};
    };
    auto read_W = [&](const char *tile, int b, int j) -> i32x8 {
        const char *p = tile + rdW + b * 64 + j * 32 * ROW_BYTES;
        const u32x4 lo = *reinterpret_cast<const u32x4 *>(p), hi = *reinterpret_cast<const u32x4 *>(p + 16);
        return i32x8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    };

    f32x16 acc[CB];
#pragma unroll
    for (int j = 0; j < CB; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;

    u32x4 rawA[2][2], rawW[2][2];
    i32x8 fw[R], fa;

    // ---- prologue: W tile 0 decoded into stage 0, A/W tile 1 in flight, first fragments in registers
    load_A(rawA[0]);
    load_W(0, rawW[0]);
    load_A(rawA[1]);
    load_W(1, rawW[1]);
    stage_W(rawW[0], 0, lds);
    stage_W(rawW[0], 1, lds);
    fa = decode_fragment<FMT_A, NWM != 8>(rawA[0][0]);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < R; ++q) fw[q] = read_W(lds, q / CB, q % CB);

    // One K step over LDS stage s: NQ = 2 CB MFMAs (block 0, then block 1).  MFMA q uses ring slot
    // q mod R, which is refilled right behind it with fragment q + R: of this step, or, from
    // q = NQ - R on, of the next step; the workgroup barrier sits before that MFMA, and the next W
    // tile is decoded into the other stage before it.  The A fragment of the next block is decoded
    // during the current one.  Every step is the same straight-line code; the last steps decode and
    // prefetch tiles of zeros.
    auto step = [&](int64_t kt, auto stage_tag) {
        constexpr int s = decltype(stage_tag)::value;
        const char *cur = lds + s * STAGE_BYTES;
        char *nxt = lds + (s ^ 1) * STAGE_BYTES;
        load_W(kt + 2, rawW[s]);
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const i32x8 fa_cur = fa;
#pragma unroll
            for (int j = 0; j < CB; ++j) {
                const int q = b * CB + j;
                if (q == NQ - R) __syncthreads();
                acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa_cur, fw[q % R], acc[j], 0, 0, 0, 0, 0, 0);
                const int qn = q + R;
                fw[q % R] = qn < NQ ? read_W(cur, qn / CB, qn % CB) : read_W(nxt, (qn - NQ) / CB, (qn - NQ) % CB);
                if (q == 0) stage_W(rawW[s ^ 1], 0, nxt);
                if (q == (NQ - R) / 2) stage_W(rawW[s ^ 1], 1, nxt);
            }
            fa = b == 0 ? decode_fragment<FMT_A, NWM != 8>(rawA[s][1]) : decode_fragment<FMT_A, NWM != 8>(rawA[s ^ 1][0]);
            if (b == 1) load_A(rawA[s]);                            // K step kt + 2; step kt's codes are decoded by now
#pragma unroll
            for (int r = 0; r < CB; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                 // DS reads
                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);                 // VALU
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
            for (int j = 0; j < CB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) red[((wr * CB + j) * 16 + v) * 64 + lane] = acc[j][v];
        }
        __syncthreads();
        if (kgp == 1) return;
#pragma unroll
        for (int j = 0; j < CB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][v] += red[((wr * CB + j) * 16 + v) * 64 + lane];
    }

    // ---- epilogue: C = acc * (sA sW) (+ bias) (ReLU), running maximum
    epilogue_strip<CB, WB>(g, acc, m0 + wr * 32, n0);
}

template <int FA, int FW, int NWM, int KG>
static void launch_cfg(const GemmArgs &g, bool conv, hipStream_t st)
{
    using G = Geom<NWM, KG>;
    const int tiles_m = (int)((g.M + G::T - 1) / G::T), tiles_n = (int)((g.N + G::T - 1) / G::T);
    const dim3 grid((unsigned)((tiles_m * tiles_n + 7) / 8 * 8)), block(G::THREADS);
    note_kernel(NWM == 8 ? DYBIT_KERNEL_F8_256 : NWM == 2 ? DYBIT_KERNEL_F8_64 : KG == 1 ? DYBIT_KERNEL_F8_128_KG1 : DYBIT_KERNEL_F8_128_KG2);
    if (conv) {
        auto k = gemm_f8_kernel<FA, FW, true, NWM, KG, kWriteBack>;
        note_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES));
        hipLaunchKernelGGL(k, grid, block, G::LDS_BYTES, st, g, tiles_m, tiles_n);
    } else {
        auto k = gemm_f8_kernel<FA, FW, false, NWM, KG, kWriteBack>;
        note_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES));
        hipLaunchKernelGGL(k, grid, block, G::LDS_BYTES, st, g, tiles_m, tiles_n);
    }
}

template <int FA, int FW>
static void launch(const GemmArgs &g, bool conv, bool large, hipStream_t st)
{
    if (large) return launch_cfg<FA, FW, 8, 1>(g, conv, st);
    const int64_t tiles = ((g.M + 127) / 128) * ((g.N + 127) / 128);
    // Few tiles: a quarter-size tile puts four times as many workgroups on the device (each decodes
    // its A rows for half as many columns, which costs less than idle compute units).
    // The "mid_tile" and "mid_kgroups" options override the choice.
    const DispatchOptions opt = dispatch_options();
    if (opt.mid_tile ? opt.mid_tile == 64 : tiles <= 128) return launch_cfg<FA, FW, 2, 2>(g, conv, st);
    const bool one = opt.mid_kgroups ? opt.mid_kgroups == 1 : tiles > 256;
    if (one) launch_cfg<FA, FW, 4, 1>(g, conv, st);
    else launch_cfg<FA, FW, 4, 2>(g, conv, st);
}

}  // namespace f8

// One translation unit per weight format (DYBIT_F8_W: 0 = 4-bit signed, 6 = 2-bit signed); the
// activation format is chosen here.
#ifndef DYBIT_F8_W
#error "compile with -DDYBIT_F8_W=0 or 6"
#endif
#define DYBIT_F8_CAT_(a, b) a##b
#define DYBIT_F8_CAT(a, b) DYBIT_F8_CAT_(a, b)
#define DYBIT_F8_WB(name) DYBIT_WB_NAME(name)                       // expands `name` before the suffix is pasted on
#define DYBIT_F8_LAUNCH DYBIT_F8_WB(DYBIT_F8_CAT(launch_gemm_f8_w, DYBIT_F8_W))

bool DYBIT_F8_LAUNCH(const GemmArgs &g, int a_bits, bool conv, bool large, hipStream_t st)
{
    constexpr int FW = DYBIT_F8_W;
    if (a_bits == 4) {
        if (g.a_signed) f8::launch<fast::F4S, FW>(g, conv, large, st);
        else f8::launch<fast::F4U, FW>(g, conv, large, st);
    } else if (a_bits == 2) {
        if (g.a_signed) f8::launch<fast::F2S, FW>(g, conv, large, st);
        else f8::launch<fast::F2U, FW>(g, conv, large, st);
    } else {
        return false;
    }
    return true;
}

}  // namespace dybit
