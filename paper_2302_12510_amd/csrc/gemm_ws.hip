// Weight-stationary DyBit matrix product for gfx950, for layers where a workgroup can keep its weights
// in the LDS of a compute unit once decoded (64 or 128 rows of W of K halves plus padding, <= 160 KiB): the
// 1 x 1 and the early 3 x 3 convolutions of a network, where M (output pixels) is huge and K is short.
// Up to N = 128 a workgroup holds the whole weight matrix; a wider N is split into groups of 64 columns,
// one per workgroup, and the workgroups of the groups walk over A side by side.
//
// The tiled kernels decode the weight tile of every K step again in every workgroup, and with a
// small K that work, the barriers around it and the half-empty 128-column tile of an N = 64 layer
// outweigh the matrix instructions.  Here a workgroup of eight waves decodes all of W into LDS once
// and then walks over 256-row slabs of A for as long as there are any (a persistent grid of at most
// two workgroups per compute unit).  After the initial barrier the waves never synchronise again:
// wave w owns rows 32 w .. 32 w + 31 of the slab and all N columns (N / 32 accumulator blocks), its
// lanes fetch and decode their own 32 codes of A per K step (two K steps ahead, as in the tiled
// kernels) and read W fragments from the resident tile.  Per K step a wave issues 4 * N / 32 MFMAs
// and decodes 32 codes per lane; nothing is decoded for columns that do not exist.
//
// Operand decoders, k order, out-of-range conventions and the epilogue are those of the tiled
// kernels (dybit_codec.h, tile_epilogue.h).  K must be a multiple of 64 (convolution: Cin).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <type_traits>

#include "dybit_codec.h"
#include "dybit_codec8.h"
#include "gemm_args.h"
#include "tile_common.h"
#include "tile_epilogue.h"

#ifndef DYBIT_WS_W
#error "compile with -DDYBIT_WS_W=<weight format id> (0: 4-bit, 2: 8-bit, 4: 6-bit, 6: 2-bit; signed)"
#endif

namespace dybit {
namespace ws {

using namespace fast;

// Waves per workgroup (32 rows each).  Eight; four in the write-back build of the two-block form, whose
// epilogue needs about 170 registers: three four-wave workgroups then share a compute unit (three waves per
// SIMD) where a single eight-wave one would fit, and the encoder of one overlaps the K loops of the others.
template <int CB, bool WB> constexpr int waves_of() { return (WB && CB == 2) ? 4 : 8; }
// Workgroups of the persistent grid per compute unit: what the weight tiles in LDS (160 KiB) and the registers
// allow (two-block form: two eight-wave workgroups at 128 registers, three four-wave ones at 168 in the
// write-back build; four-block form: one).
template <int CB> inline int workgroups_per_cu(int lds_bytes)
{
    const int by_lds = (160 * 1024) / lds_bytes;
    const int by_regs = CB == 2 ? (kWriteBack ? 3 : 2) : 1;
    return by_lds < by_regs ? (by_lds < 1 ? 1 : by_lds) : by_regs;
}

// N > 32 CB: the columns are split into groups of 32 CB and a workgroup keeps the weights of one group.  The
// workgroups that walk over the same slabs of A, one per group, sit on the same XCD (workgroup ids that agree
// modulo 8) and next to each other in its launch order, so that a slab read by the first comes out of that XCD's
// L2 for the others.  walker: which slab sequence this workgroup follows, of `walkers` (gridDim.x / groups).
struct ColumnGroup {
    int n0, walker, walkers;
};
template <int CB> __device__ __forceinline__ ColumnGroup column_group(int groups)
{
    ColumnGroup c{0, (int)blockIdx.x, (int)gridDim.x};
    if (groups > 1) {
        const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
        c.n0 = (local % groups) * (CB * 32);
        c.walker = (local / groups) * 8 + xcd;
        c.walkers = (int)gridDim.x / groups;
    }
    return c;
}
// Persistent grid for `groups` column groups: a multiple of 8 * groups workgroups (0: more groups than the chip
// holds workgroups), no more walkers than there are slabs (rounded up to the eight XCDs).
inline int grid_for_groups(int slabs, int groups, int resident)
{
    if (groups == 1) return slabs < resident ? slabs : resident;
    const int per = 8 * groups;
    int walkers = resident / per * 8;
    const int needed = (slabs + 7) / 8 * 8;
    if (needed < walkers) walkers = needed;
    return walkers * groups;
}

// CONV: 0 matrix product; 1 convolution whose 64-code k groups lie inside one filter tap (Cin a
// multiple of 64); 2 (ROWS) convolution with few channels where one filter row is exactly one 32-code
// run (kw * Cin = 32): the run of lane-half kq in K step t is filter row 2 t + kq of the lane's output
// pixel, fetched as aligned words and shifted / masked when it is decoded (as in the 128 x 128 kernel).
// CB: 32-column blocks per wave (N <= 32 CB).  With two blocks a wave needs few registers and two
// workgroups share a compute unit (four waves per SIMD) when their weight tiles both fit its LDS.
constexpr int ROWS = 2;

template <int FMT_A, int FMT_W, int CONV, int CB, bool WB>
__global__ __launch_bounds__((64 * waves_of<CB, WB>()), (CB == 2 ? (WB ? 3 : 4) : 2)) void gemm_ws_kernel(const GemmArgs g, const int slabs, const int row_bytes, const int groups)
{
    constexpr int THREADS = 64 * waves_of<CB, WB>(), SLAB = 32 * waves_of<CB, WB>();
    using CA = Codec<FMT_A>;
    using CW = Codec<FMT_W>;
    constexpr int WORDS_A = CA::BITS;                               // 32-bit words in a run of 32 codes
    constexpr int NA = CONV == ROWS ? (WORDS_A + 1 + 3) / 4 : (CA::BITS + 3) / 4, NW = (CW::BITS + 3) / 4;
    constexpr int RUN_A = 4 * CA::BITS, RUN_W = 4 * CW::BITS;       // bytes of a run of 32 codes
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kq = lane >> 5;
    const int ktiles = (int)(g.K / 64);
    const ColumnGroup cg = column_group<CB>(groups);

    // ROWS reads aligned words; the dispatcher takes it only for tensors of a whole number of words
    const __amdgpu_buffer_rsrc_t rsrcA = code_descriptor(g.A, g.a_bytes), rsrcW = code_descriptor(g.W, g.w_bytes);

    // ---- W: every run of 32 codes is decoded once and stays.  Row n of the tile is K halves plus 16
    // bytes of padding (fragment reads of 32 consecutive rows then fall into different banks); rows
    // N .. 32 CB - 1 hold zeros (their runs are fetched from the out-of-range offset).
    {
        const int runs_per_row = ktiles * 2, w_row_bytes = (int)(g.K * CW::BITS / 8);
        const int total = CB * 32 * runs_per_row;
        for (int r = tid; r < total; r += THREADS) {
            const int row = r / runs_per_row, run = r - row * runs_per_row;
            u32x4 raw[NW];
            load_run<CW::BITS>(rsrcW, cg.n0 + row < g.N ? (u32)((cg.n0 + row) * w_row_bytes + run * RUN_W) : kOob, raw);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                u32 d[4];
                decode_eight<FMT_W>(raw, q, d);
                *reinterpret_cast<u32x4 *>(lds + row * row_bytes + run * 64 + q * 16) = u32x4{d[0], d[1], d[2], d[3]};
            }
        }
    }
    __syncthreads();

    const int a_row_bytes = (int)(g.K * CA::BITS / 8);
    const int pix_bytes = CONV ? g.pix_bytes : 0;
    const u32 rdW = (u32)(lane & 31) * (u32)row_bytes + (u32)kq * 64;   // K step adds 128 B, block kk 16 B, column block j 32 rows

    float run_max = 0.0f;                                            // max |C| over every strip this lane stores
    for (int slab = cg.walker; slab < slabs; slab += cg.walkers) {
        const int64_t m_strip = (int64_t)slab * SLAB + wave * 32;
        if (m_strip >= g.M) continue;                                // uniform per wave; no barriers below
        // ---- A: the lane's own row, the 32 codes kq of every K step
        u32 offA;
        int hi0 = 0, wi0 = 0;
        bool okA;
        u32 row_keep[CONV == ROWS ? WORDS_A : 1];                    // ROWS: bits of a run that belong to taps inside the image
        {
            const int64_t m = m_strip + (lane & 31);
            okA = m < g.M;
            if (CONV) {
                // M fits 31 bits (checked at launch): 32-bit divisions, a fraction of the cost of 64-bit ones,
                // and this set-up runs once per slab, which for a short K is as much work as the K loop
                const u32 mm = okA ? (u32)m : 0u;
                const u32 plane = (u32)g.Ho * (u32)g.Wo;
                const int b = (int)(mm / plane);
                const int rem = (int)(mm - (u32)b * plane);
                const int ho = (int)((u32)rem / (u32)g.Wo), wo = rem - ho * g.Wo;
                hi0 = ho * g.stride - g.pad;
                wi0 = wo * g.stride - g.pad;
                if (CONV == ROWS) {
                    offA = (u32)(((b * g.H + hi0) * g.Wd + wi0) * pix_bytes);   // first byte of filter row 0 (may be negative); the image is under 2 GiB
                    const int taps = g.kw, tap_bits = g.Cin * CA::BITS;                       // kw * Cin = 32
                    const int t_lo = max(0, -wi0), t_hi = max(min(taps, g.Wd - wi0), t_lo);
#pragma unroll
                    for (int i = 0; i < WORDS_A; ++i) {
                        // bits [lo, up) of word i, 0 <= lo <= up <= 32
                        const int lo = min(max(t_lo * tap_bits - 32 * i, 0), 32), up = min(max(t_hi * tap_bits - 32 * i, 0), 32);
                        const u32 below_up = up >= 32 ? ~0u : (1u << up) - 1u, below_lo = lo >= 32 ? ~0u : (1u << lo) - 1u;
                        row_keep[i] = below_up & ~below_lo;
                    }
                } else {
                    offA = (u32)(((b * g.H + hi0) * g.Wd + wi0) * pix_bytes + kq * RUN_A);   // the image is under 2 GiB
                }
            } else {
                offA = okA ? (u32)(m * a_row_bytes + kq * RUN_A) : kOob;
            }
        }
        // position of the next K step to load: first k, and for a convolution its filter row, filter
        // column and first channel (uniform over the wave), counted up from step to step
        int a_k0 = 0;
        TapCounter tap;
        auto load_A = [&](u32x4 *raw) {
            if constexpr (CONV == ROWS) {
                const int fr = (a_k0 >> 5) + kq;
                const int hi = hi0 + fr;
                const bool in = okA && a_k0 < g.K && (unsigned)hi < (unsigned)g.H;
                const int byte_off = (int)offA + fr * g.Wd * pix_bytes;
                const int shift = byte_off & 3, base = byte_off - shift;
                u32 w[NA * 4];
#pragma unroll
                for (int j = 0; j < NA * 4; ++j) w[j] = 0;
#pragma unroll
                for (int j = 0; j <= WORDS_A; ++j) {
                    const int o = base + 4 * j;                  // a word before the tensor is "outside" explicitly
                    w[j] = __builtin_amdgcn_raw_buffer_load_b32(rsrcA, (in && o >= 0) ? (u32)o : kOob, 0, 0);
                }
                w[NA * 4 - 1] = (u32)shift;                      // travels with the words to the decoder
#pragma unroll
                for (int p = 0; p < NA; ++p) raw[p] = u32x4{w[4 * p], w[4 * p + 1], w[4 * p + 2], w[4 * p + 3]};
                a_k0 += 64;
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
            a_k0 += 64;
            if (CONV == 1) {
                tap.advance(64, g);
            }
        };
        auto decode_A = [&](const u32x4 *raw, int q) -> f16x8 {
            u32 d[4];
            if constexpr (CONV == ROWS) {
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

        f32x16 acc[CB];
#pragma unroll
        for (int j = 0; j < CB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;

        u32x4 rawA[2][NA];
        load_A(rawA[0]);
        load_A(rawA[1]);
        f16x8 fa = decode_A(rawA[0], 0);

        // One K step: four k blocks of CB MFMAs; the A fragment of the next block is decoded while
        // this block's MFMAs run, the codes of K step kt + 2 are requested once step kt's are decoded.
        auto step = [&](int kt, auto stage_tag) {
            constexpr int s = decltype(stage_tag)::value;
            const char *wk = lds + rdW + kt * 128;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const f16x8 fa_cur = fa;
                f16x8 fw[CB];
#pragma unroll
                for (int j = 0; j < CB; ++j) fw[j] = *reinterpret_cast<const f16x8 *>(wk + kk * 16 + j * 32 * row_bytes);
                fa = kk < 3 ? decode_A(rawA[s], kk + 1) : decode_A(rawA[s ^ 1], 0);
#pragma unroll
                for (int j = 0; j < CB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa_cur, fw[j], acc[j], 0, 0, 0);
                if (kk == 3) load_A(rawA[s]);
            }
        };
        for (int kt = 0; kt < ktiles; kt += 2) {
            step(kt, std::integral_constant<int, 0>{});
            if (kt + 1 < ktiles) step(kt + 1, std::integral_constant<int, 1>{});
        }
        run_max = fmaxf(run_max, epilogue_strip<CB, WB, false, CA::ACC_EXP + CW::ACC_EXP>(g, acc, m_strip, cg.n0));
    }

    // ---- running maximum: one merge per workgroup.  The persistent waves finish their strips in step,
    // so a merge per strip would send thousands of waves to the same word at the same moment.
    if (g.absmax_bits) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) run_max = fmaxf(run_max, __shfl_xor(run_max, off, 64));
        __syncthreads();                                            // every wave is done with the weight tile
        float *red = reinterpret_cast<float *>(lds);
        if (lane == 0) red[wave] = run_max;
        __syncthreads();
        if (tid == 0) {
            float m = red[0];
#pragma unroll
            for (int w = 1; w < THREADS / 64; ++w) m = fmaxf(m, red[w]);
            const uint32_t bits = __float_as_uint(m);
            if (bits > __hip_atomic_load(g.absmax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(g.absmax_bits, bits);
        }
    }
}

// ---------------------------------------------------------------------------
// The same kernel on the fp8 matrix path, for pairs of 4- and 2-bit formats (every value exact in e4m3,
// dybit_codec8.h): `v_mfma_f32_32x32x64_f8f6f4` contracts 64 k per instruction in the time the fp16 instruction
// needs for 32, the resident weight tile holds bytes instead of halves (half the LDS, half the bytes per
// fragment read: with one fragment read per MFMA, LDS bandwidth is what the fp16 form runs into at N = 64),
// and a K step is one MFMA per column block.  Lane (row, kq) supplies k = 32 kq .. + 31 of the step: one
// 128-bit (2-bit codes: 64-bit) load of its own row, decoded in registers into the 32-byte A fragment.
// CONV: 0 matrix product, 1 convolution with Cin a multiple of 64.
// ---------------------------------------------------------------------------
#if DYBIT_WS_W == 0 || DYBIT_WS_W == 6
template <int FMT_A, int FMT_W, int CONV, int CB, bool WB>
__global__ __launch_bounds__((64 * waves_of<CB, WB>()), (CB == 2 ? (WB ? 3 : 4) : 2)) void gemm_ws8_kernel(const GemmArgs g, const int slabs, const int row_bytes, const int groups)
{
    constexpr int THREADS = 64 * waves_of<CB, WB>(), SLAB = 32 * waves_of<CB, WB>();
    using f8::i32x8;
    constexpr int BA = f8::bits_of<FMT_A>(), BW = f8::bits_of<FMT_W>();
    constexpr int RUN_A = 4 * BA, RUN_W = 4 * BW;                    // bytes of a run of 32 codes
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kq = lane >> 5;
    const int ktiles = (int)(g.K / 64);
    const ColumnGroup cg = column_group<CB>(groups);
    const __amdgpu_buffer_rsrc_t rsrcA = code_descriptor(g.A, g.a_bytes), rsrcW = code_descriptor(g.W, g.w_bytes);
    auto load_run8 = [&](const __amdgpu_buffer_rsrc_t &rs, u32 off, auto bits_tag) -> u32x4 {
        if constexpr (decltype(bits_tag)::value == 2) {
            const f8::u32x2 two = __builtin_amdgcn_raw_buffer_load_b64(rs, off, 0, 0);
            return u32x4{two.x, two.y, 0u, 0u};
        } else {
            return __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
        }
    };

    // ---- W: every run of 32 codes is decoded once into 32 bytes and stays.  Row n of the tile is K bytes plus
    // 16 bytes of padding; rows N .. 32 CB - 1 hold zeros (fetched from the out-of-range offset).
    {
        const int runs_per_row = ktiles * 2, w_row_bytes = (int)(g.K * BW / 8);
        const int total = CB * 32 * runs_per_row;
        for (int r = tid; r < total; r += THREADS) {
            const int row = r / runs_per_row, run = r - row * runs_per_row;
            const u32x4 raw = load_run8(rsrcW, cg.n0 + row < g.N ? (u32)((cg.n0 + row) * w_row_bytes + run * RUN_W) : kOob, std::integral_constant<int, BW>{});
            const i32x8 f = f8::decode_fragment<FMT_W>(raw);
            char *dst = lds + row * row_bytes + run * 32;
            *reinterpret_cast<u32x4 *>(dst) = u32x4{(u32)f[0], (u32)f[1], (u32)f[2], (u32)f[3]};
            *reinterpret_cast<u32x4 *>(dst + 16) = u32x4{(u32)f[4], (u32)f[5], (u32)f[6], (u32)f[7]};
        }
    }
    __syncthreads();

    const int a_row_bytes = (int)(g.K * BA / 8);
    const int pix_bytes = CONV ? g.pix_bytes : 0;
    const u32 rdW = (u32)(lane & 31) * (u32)row_bytes + (u32)kq * 32;   // K step adds 64 B, column block j 32 rows

    float run_max = 0.0f;
    for (int slab = cg.walker; slab < slabs; slab += cg.walkers) {
        const int64_t m_strip = (int64_t)slab * SLAB + wave * 32;
        if (m_strip >= g.M) continue;                                // uniform per wave; no barriers below
        u32 offA;
        int hi0 = 0, wi0 = 0;
        const int64_t m = m_strip + (lane & 31);
        const bool okA = m < g.M;
        if (CONV) {
            const PixelOrigin o = pixel_origin(g, okA ? m : 0);
            hi0 = o.hi0;
            wi0 = o.wi0;
            offA = (u32)(o.first_pixel * pix_bytes + kq * RUN_A);    // the image is under 2 GiB
        } else {
            offA = okA ? (u32)(m * a_row_bytes + kq * RUN_A) : kOob;
        }
        int a_k0 = 0;
        TapCounter tap;
        auto load_A = [&]() -> u32x4 {
            u32 off;
            if (CONV) {
                const bool in = okA && a_k0 < g.K && tap.inside(g, hi0, wi0);
                off = in ? offA + (u32)tap.byte_offset(g, pix_bytes, BA) : kOob;   // padding reads code 0
                tap.advance(64, g);
            } else {
                off = a_k0 < g.K ? offA + (u32)(a_k0 * BA / 8) : kOob;
            }
            a_k0 += 64;
            return load_run8(rsrcA, off, std::integral_constant<int, BA>{});
        };

        f32x16 acc[CB];
#pragma unroll
        for (int j = 0; j < CB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;

        u32x4 rawA[2];
        rawA[0] = load_A();
        rawA[1] = load_A();
        i32x8 fa = f8::decode_fragment<FMT_A, true>(rawA[0]);
        // One K step: CB MFMAs on the fragment decoded during the previous step; the codes of step kt + 2 are
        // requested once step kt + 1's are decoded.
        auto step = [&](int kt, auto stage_tag) {
            constexpr int s = decltype(stage_tag)::value;
            const char *wk = lds + rdW + kt * 64;
            const i32x8 fa_cur = fa;
            i32x8 fw[CB];
#pragma unroll
            for (int j = 0; j < CB; ++j) {
                const u32x4 lo = *reinterpret_cast<const u32x4 *>(wk + j * 32 * row_bytes);
                const u32x4 hi = *reinterpret_cast<const u32x4 *>(wk + j * 32 * row_bytes + 16);
                fw[j] = i32x8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
            }
            fa = f8::decode_fragment<FMT_A, true>(rawA[s ^ 1]);
#pragma unroll
            for (int j = 0; j < CB; ++j)
                acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa_cur, fw[j], acc[j], 0, 0, 0, 0, 0, 0);
            rawA[s] = load_A();
        };
        for (int kt = 0; kt < ktiles; kt += 2) {
            step(kt, std::integral_constant<int, 0>{});
            if (kt + 1 < ktiles) step(kt + 1, std::integral_constant<int, 1>{});
        }
        run_max = fmaxf(run_max, epilogue_strip<CB, WB, false, 0>(g, acc, m_strip, cg.n0));
    }

    if (g.absmax_bits) {                                            // one merge per workgroup, as in the fp16 form
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) run_max = fmaxf(run_max, __shfl_xor(run_max, off, 64));
        __syncthreads();                                            // every wave is done with the weight tile
        float *red = reinterpret_cast<float *>(lds);
        if (lane == 0) red[wave] = run_max;
        __syncthreads();
        if (tid == 0) {
            float mm = red[0];
#pragma unroll
            for (int w = 1; w < THREADS / 64; ++w) mm = fmaxf(mm, red[w]);
            const uint32_t bits = __float_as_uint(mm);
            if (bits > __hip_atomic_load(g.absmax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(g.absmax_bits, bits);
        }
    }
}

template <int FA, int FW, int CONV, int CB>
static bool launch_cb8(const GemmArgs &g, hipStream_t st, int row_bytes, int lds_bytes)
{
    constexpr int THREADS = 64 * waves_of<CB, kWriteBack>(), SLAB = 32 * waves_of<CB, kWriteBack>();
    const int slabs = (int)((g.M + SLAB - 1) / SLAB);
    const int groups = (int)((g.N + CB * 32 - 1) / (CB * 32));
    const int grid = grid_for_groups(slabs, groups, 256 * workgroups_per_cu<CB>(lds_bytes));
    if (grid < 1) return false;
    auto k = gemm_ws8_kernel<FA, FW, CONV, CB, kWriteBack>;
    note_kernel(DYBIT_KERNEL_F8_WS);
    note_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
    hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3(THREADS), lds_bytes, st, g, slabs, row_bytes, groups);
    return true;
}
#endif

template <int FA, int FW, int CONV, int CB>
static bool launch_cb(const GemmArgs &g, hipStream_t st, int row_bytes, int lds_bytes)
{
    constexpr int THREADS = 64 * waves_of<CB, kWriteBack>(), SLAB = 32 * waves_of<CB, kWriteBack>();
    const int slabs = (int)((g.M + SLAB - 1) / SLAB);
    const int groups = (int)((g.N + CB * 32 - 1) / (CB * 32));
    const int grid = grid_for_groups(slabs, groups, 256 * workgroups_per_cu<CB>(lds_bytes));
    if (grid < 1) return false;
    auto k = gemm_ws_kernel<FA, FW, CONV, CB, kWriteBack>;
    note_kernel(DYBIT_KERNEL_F16_WS);
    note_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
    hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3(THREADS), lds_bytes, st, g, slabs, row_bytes, groups);
    return true;
}

template <int FA, int FW>
static bool launch(const GemmArgs &g, bool conv, hipStream_t st)
{
    // Up to 128 columns a wave takes all of them (two or four 32-column blocks): with more, its accumulators
    // leave no registers for the epilogue.  Beyond that the columns go in groups of 64, one group per workgroup.
    const int cb = (g.N <= 64 || g.N > 128) ? 2 : 4;
    const bool rows = conv && g.Cin < 64;                            // kw * Cin = 32 (checked by the dispatcher)
    if (g.M > 0x7fffffff) return false;
#if DYBIT_WS_W == 0 || DYBIT_WS_W == 6
    // both operands 4- or 2-bit: the fp8 matrix path, unless the "gemm_mfma" option asks for fp16
    if constexpr (FA == F4S || FA == F4U || FA == F2S || FA == F2U) {
        const int row8 = (int)g.K + 16, lds8 = cb * 32 * row8;
        if (!rows && !dispatch_options().mfma_f16 && lds8 <= 160 * 1024) {
            if (cb == 2) return conv ? launch_cb8<FA, FW, 1, 2>(g, st, row8, lds8) : launch_cb8<FA, FW, 0, 2>(g, st, row8, lds8);
            return conv ? launch_cb8<FA, FW, 1, 4>(g, st, row8, lds8) : launch_cb8<FA, FW, 0, 4>(g, st, row8, lds8);
        }
    }
#endif
    const int row_bytes = (int)g.K * 2 + 16;
    const int lds_bytes = cb * 32 * row_bytes;
    if (lds_bytes > 160 * 1024) return false;
#define DYBIT_WS_CB(C_) \
    return rows ? launch_cb<FA, FW, ROWS, C_>(g, st, row_bytes, lds_bytes) \
         : conv ? launch_cb<FA, FW, 1, C_>(g, st, row_bytes, lds_bytes) \
                : launch_cb<FA, FW, 0, C_>(g, st, row_bytes, lds_bytes)
    if (cb == 2) { DYBIT_WS_CB(2); }
    DYBIT_WS_CB(4);
#undef DYBIT_WS_CB
}

}  // namespace ws

// One translation unit per weight format (compile time); the entry point's name carries it.
// Returns false when the weight matrix does not fit the LDS of a compute unit.
#define DYBIT_WS_NAME2(w) DYBIT_WB_NAME(launch_gemm_ws_w##w)
#define DYBIT_WS_NAME(w) DYBIT_WS_NAME2(w)
bool DYBIT_WS_NAME(DYBIT_WS_W)(const GemmArgs &g, int a_bits, bool conv, hipStream_t st)
{
    using namespace fast;
    const int fa = (a_bits == 8 ? F8S : a_bits == 6 ? F6S : a_bits == 2 ? F2S : F4S) + (g.a_signed ? 0 : 1);
    switch (fa) {
        case F2S: return ws::launch<F2S, DYBIT_WS_W>(g, conv, st);
        case F2U: return ws::launch<F2U, DYBIT_WS_W>(g, conv, st);
        case F4S: return ws::launch<F4S, DYBIT_WS_W>(g, conv, st);
        case F4U: return ws::launch<F4U, DYBIT_WS_W>(g, conv, st);
        case F6S: return ws::launch<F6S, DYBIT_WS_W>(g, conv, st);
        case F6U: return ws::launch<F6U, DYBIT_WS_W>(g, conv, st);
        case F8S: return ws::launch<F8S, DYBIT_WS_W>(g, conv, st);
        case F8U: return ws::launch<F8U, DYBIT_WS_W>(g, conv, st);
        default: return false;
    }
}

}  // namespace dybit
