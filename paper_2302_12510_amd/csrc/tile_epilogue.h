// Epilogue shared by the tiled matrix-product kernels: C = acc * (sA sW) (+ bias) (+ residual) (ReLU),
// sW the scale of the weight tensor or of the output column's weight row (g.w_per_channel),
// optional running maximum of |C|, optional write-back of C as DyBit codes (Sec. III-B), for the
// 32-row strip of accumulator blocks one wave holds.
//
// Accumulator v of a lane is row 8 (v / 4) + 4 (lane / 32) + v % 4 and column lane % 32 of its
// 32 x 32 block.  The strip is stored through a buffer descriptor that starts at the strip's first
// row and ends after its last valid row, with 32-bit byte offsets: a row past M falls outside the
// descriptor and a column past N gets an offset of 2^31, so the hardware drops those stores and the
// loop needs neither 64-bit address arithmetic nor per-element branches.
#ifndef DYBIT_TILE_EPILOGUE_H
#define DYBIT_TILE_EPILOGUE_H

#include "../../include/dybit.h"
#include "dybit_codec.h"
#include "gemm_args.h"
#include "requant.h"

namespace dybit {

// ACC_EXP: the accumulators hold the sum times 2^-ACC_EXP (operands decoded on a power-of-two scale,
// dybit_codec.h); they are multiplied back first, which is exact, so the result is rounded as before.
template <int ACC_EXP>
__device__ __forceinline__ float acc_value(float a)
{
    if constexpr (ACC_EXP == 0) return a;
    else return a * __uint_as_float((uint32_t)(127 + ACC_EXP) << 23);
}

template <int CB, bool HAS_RES, int ACC_EXP>
__device__ __forceinline__ float store_strip(const GemmArgs &g, const fast::f32x16 (&acc)[CB], const int64_t m_strip,
                                             const int64_t n0, const int rows, const float alpha)
{
    const int lane = threadIdx.x & 63, kq = lane >> 5;
    // The variants of this function are the sides of one branch and derive the same columns, bias
    // values and store offsets from the lane number.  Without this barrier the compiler computes
    // all of them once above the branch (128 offsets per lane), where they do not fit the register
    // file beside the accumulators and are spilled.
    int col = lane & 31;
    asm volatile("" : "+v"(col));
    const uint32_t ldc4 = (uint32_t)g.ldc * 4u;
    const int records = (int)((uint32_t)rows * ldc4);
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(g.C + m_strip * g.ldc, 0, records, 0x00020000);
    const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(HAS_RES ? g.residual + m_strip * g.ldc : g.C), 0, HAS_RES ? records : 0, 0x00020000);
    const bool track = g.absmax_bits != nullptr;
    float mx = 0.0f;
    // The shortcut values of block j + 1 are requested before block j is stored (kernels with at most
    // four blocks per wave: the others have no registers to spare).  Memory operations retire in order,
    // so waiting for those loads does not wait for the stores issued after them; without the prefetch
    // every block's loads queue behind the previous block's stores and the two latencies add up.
    constexpr bool PREFETCH = HAS_RES && CB <= 4;
    auto first_offset = [&](int j, bool &n_ok, int64_t &n) {
        n = n0 + j * 32 + col;
        n_ok = n < g.N;
        return (n_ok ? (uint32_t)n * 4u : 0x80000000u) + (uint32_t)(4 * kq) * ldc4;
    };
    auto load_shortcut = [&](uint32_t off, float (&r)[16]) {           // out-of-range elements read 0
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            r[v] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rres, off, 0, 0));
            off += (v & 3) == 3 ? 5u * ldc4 : ldc4;
        }
    };
    float res2[2][16];
    if (PREFETCH) {
        bool ok0; int64_t nn0;
        load_shortcut(first_offset(0, ok0, nn0), res2[0]);
    }
#pragma unroll
    for (int j = 0; j < CB; ++j) {
        bool n_ok; int64_t n;
        const uint32_t off0 = first_offset(j, n_ok, n);
        const float b = (g.bias && n_ok) ? g.bias[n] : 0.0f;
        const float al = g.w_per_channel ? alpha * g.w_scale[n_ok ? n : 0] : alpha;
        float (&res)[16] = res2[PREFETCH ? (j & 1) : 0];
        if (HAS_RES && !PREFETCH) load_shortcut(off0, res);
        if (PREFETCH && j + 1 < CB) {
            bool ok1; int64_t nn1;
            load_shortcut(first_offset(j + 1, ok1, nn1), res2[(j + 1) & 1]);
        }
        uint32_t off = off0;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float c = acc_value<ACC_EXP>(acc[j][v]) * al + b;
            if (HAS_RES) c += res[v];
            if (g.relu) c = fmaxf(c, 0.0f);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(c), rsrc, off, 0, 2);
            if (track) {
                // a row past M holds bias only (its codes read as zeros): keep it out of the maximum
                const int r = 8 * (v >> 2) + 4 * kq + (v & 3);
                mx = fmaxf(mx, (n_ok && r < rows) ? fabsf(c) : 0.0f);
            }
            off += (v & 3) == 3 ? 5u * ldc4 : ldc4;                     // rows 0-3, 8-11, 16-19, 24-27 (+ 4 kq)
        }
    }
    return mx;
}

// The same strip with the write-back encoder (requant.h): per 32 x 32 block, three phases over the
// lane's values (eight at a time) so that the instruction streams of the values interleave and the only branch is
// one per block -- (1) result, optional fp32 store, rounded real-valued code; (2) only if some
// lane's value sits within 2^-G of a decision point: the exact decision for those;
// (3) sign, packing across lanes, store of the packed words through a descriptor of their own.
// A NULL fp32 output becomes an empty descriptor whose stores the hardware drops.
template <int CB, bool HAS_RES, int BITS, int ACC_EXP>
__device__ __forceinline__ float store_strip_wb(const GemmArgs &g, const fast::f32x16 (&acc)[CB], const int64_t m_strip,
                                                const int64_t n0, const int rows, const float alpha)
{
    const int lane = threadIdx.x & 63, kq = lane >> 5;
    int col = lane & 31;
    asm volatile("" : "+v"(col));                                      // see store_strip
    const uint32_t ldc4 = (uint32_t)g.ldc * 4u;
    const int records = (int)((uint32_t)rows * ldc4);
    float *const c_base = g.C ? g.C + m_strip * g.ldc : const_cast<float *>(g.a_scale);
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(c_base, 0, g.C ? records : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(HAS_RES ? g.residual + m_strip * g.ldc : g.a_scale), 0, HAS_RES ? records : 0, 0x00020000);
    const uint32_t qrow = (uint32_t)g.q_row_bytes;
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(g.q_out + m_strip * g.q_row_bytes, 0,
                                                                        (int)((uint32_t)rows * qrow), 0x00020000);
    const Requant rqp = make_requant(g.q_scale, BITS, g.q_signed);
    if (!rqp.ok && m_strip == 0 && n0 == 0 && lane == 0) *g.async_error = DYBIT_ERR_BAD_SCALE;   // no codes, flag the call
    constexpr int GV = 8;
    const bool track = g.absmax_bits != nullptr;
    // ReLU as a maximum with a uniform floor (no select per value).  Without ReLU the floor is NaN:
    // the maximum of a number and NaN is the number, and a NaN result stays NaN (and becomes code 0)
    const float relu_floor = g.relu ? 0.0f : __builtin_nanf("");
    float mx = 0.0f;
    constexpr bool PREFETCH = HAS_RES && CB <= 4;
    float res2[2][GV];
    uint32_t roff = 0;                                                  // walks the shortcut's rows like `off` walks C's
    auto load_shortcut = [&](int first_v, float (&r)[GV]) {
#pragma unroll
        for (int u = 0; u < GV; ++u) {
            r[u] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rres, roff, 0, 0));
            roff += ((first_v + u) & 3) == 3 ? 5u * ldc4 : ldc4;
        }
    };
#pragma unroll
    for (int j = 0; j < CB; ++j) {
        const int64_t n = n0 + j * 32 + col;
        const bool n_ok = n < g.N;
        const float b = (g.bias && n_ok) ? g.bias[n] : 0.0f;
        const float al = g.w_per_channel ? alpha * g.w_scale[n_ok ? n : 0] : alpha;
        const uint32_t off0 = (n_ok ? (uint32_t)n * 4u : 0x80000000u) + (uint32_t)(4 * kq) * ldc4;
        const PackSlot slot = pack_slot<BITS>(lane, (uint32_t)n);
        uint32_t qoff = ((n_ok && slot.stores && rqp.ok) ? slot.byte_off : 0x80000000u) + (uint32_t)(4 * kq) * qrow;
        uint32_t off = off0;
        if (HAS_RES && (j == 0 || !PREFETCH)) { roff = off0; if (PREFETCH) load_shortcut(0, res2[0]); }
#pragma unroll
        for (int h = 0; h < 16; h += GV) {                                   // GV values at a time: fewer live registers
            // the shortcut values of the next group are requested before this group is stored (see
            // store_strip) where the kernel has registers for them; else they are loaded here
            const int grp = (j * 16 + h) / GV;
            float (&res)[GV] = res2[PREFETCH ? (grp & 1) : 0];
            if (HAS_RES && !PREFETCH) load_shortcut(h, res);
            if (PREFETCH) {
                if (h + GV < 16) {
                    load_shortcut(h + GV, res2[(grp + 1) & 1]);
                } else if (j + 1 < CB) {
                    const int64_t n1 = n0 + (j + 1) * 32 + col;
                    roff = (n1 < g.N ? (uint32_t)n1 * 4u : 0x80000000u) + (uint32_t)(4 * kq) * ldc4;
                    load_shortcut(0, res2[(grp + 1) & 1]);
                }
            }
            float c[GV];
            uint32_t zb[GV];
            uint32_t settle_key = 0xffffffffu;                               // minimum over the values: 0 = some value needs phase 2
#pragma unroll
            for (int u = 0; u < GV; ++u) {                                   // phase 1
                const int v = h + u;
                c[u] = acc_value<ACC_EXP>(acc[j][v]) * al + b;
                if (HAS_RES) c[u] += res[u];
                c[u] = fmaxf(c[u], relu_floor);
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(c[u]), rsrc, off, 0, 2);
                off += (v & 3) == 3 ? 5u * ldc4 : ldc4;
                if (track) {
                    const int r = 8 * (v >> 2) + 4 * kq + (v & 3);
                    mx = fmaxf(mx, (n_ok && r < rows) ? fabsf(c[u]) : 0.0f);
                }
                zb[u] = requant_rounded(c[u], rqp);
                settle_key = min(settle_key, requant_settle_key(zb[u]));
            }
            uint32_t code[GV];
#pragma unroll
            for (int u = 0; u < GV; ++u) code[u] = requant_magnitude(zb[u], rqp);
            if (__builtin_amdgcn_ballot_w64(settle_key == 0u)) {             // phase 2 (uniform branch)
#pragma unroll
                for (int u = 0; u < GV; ++u) {
                    const uint32_t fixed = requant_settle(c[u], code[u], rqp);
                    code[u] = requant_needs_settling(zb[u]) ? fixed : code[u];
                }
            }
            if (rqp.is_signed) {                                             // uniform
#pragma unroll
                for (int u = 0; u < GV; ++u) code[u] = requant_with_sign(code[u], c[u], rqp);
            }
#pragma unroll
            for (int u = 0; u < GV; ++u) {                                   // phase 3
                const uint32_t packed = pack_word<BITS>(code[u], lane, slot);
                if constexpr (BITS == 6) __builtin_amdgcn_raw_buffer_store_b32(packed, rq, qoff, 0, 2);
                else __builtin_amdgcn_raw_buffer_store_b8((unsigned char)packed, rq, qoff, 0, 2);
                qoff += ((h + u) & 3) == 3 ? 5u * qrow : qrow;
            }
        }
    }
    return mx;
}

// WB: the kernel is the write-back build (codes are written, see requant.h); kernels are compiled
// in both forms so that the plain form carries none of the encoder's registers or branches.
// FOLD: merge the strip's maximum into the running maximum here (one read, at most one atomic per
// wave); a kernel whose waves store many strips passes false, keeps the returned per-lane maximum
// and merges once at its end.
template <int CB, bool WB, bool FOLD = true, int ACC_EXP = 0>
__device__ __forceinline__ float epilogue_strip(const GemmArgs &g, const fast::f32x16 (&acc)[CB],
                                               const int64_t m_strip, const int64_t n0)
{
    const int lane = threadIdx.x & 63, kq = lane >> 5;
    const float alpha = g.w_per_channel ? *g.a_scale : (*g.a_scale) * (*g.w_scale);   // per channel: sW[n] joins per column
    const int64_t rows_left = g.M - m_strip;                       // uniform over the wave
    const int rows = rows_left >= 32 ? 32 : rows_left > 0 ? (int)rows_left : 0;
    float mx = 0.0f;
    if (WB) {                                                       // the host has checked ldc, N and the format
        if (g.residual) {
            mx = g.q_bits == 4 ? store_strip_wb<CB, true, 4, ACC_EXP>(g, acc, m_strip, n0, rows, alpha)
               : g.q_bits == 8 ? store_strip_wb<CB, true, 8, ACC_EXP>(g, acc, m_strip, n0, rows, alpha)
                               : store_strip_wb<CB, true, 6, ACC_EXP>(g, acc, m_strip, n0, rows, alpha);
        } else {
            mx = g.q_bits == 4 ? store_strip_wb<CB, false, 4, ACC_EXP>(g, acc, m_strip, n0, rows, alpha)
               : g.q_bits == 8 ? store_strip_wb<CB, false, 8, ACC_EXP>(g, acc, m_strip, n0, rows, alpha)
                               : store_strip_wb<CB, false, 6, ACC_EXP>(g, acc, m_strip, n0, rows, alpha);
        }
    } else if (g.ldc < (1 << 23)) {
        mx = g.residual ? store_strip<CB, true, ACC_EXP>(g, acc, m_strip, n0, rows, alpha)
                        : store_strip<CB, false, ACC_EXP>(g, acc, m_strip, n0, rows, alpha);
    } else {                                                        // leading dimension too large for 32-bit offsets
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            const int64_t n = n0 + j * 32 + (lane & 31);
            const bool n_ok = n < g.N;
            const float b = (g.bias && n_ok) ? g.bias[n] : 0.0f;
            const float al = g.w_per_channel ? alpha * g.w_scale[n_ok ? n : 0] : alpha;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = 8 * (v >> 2) + 4 * kq + (v & 3);
                if (n_ok && r < rows) {
                    float c = acc_value<ACC_EXP>(acc[j][v]) * al + b;
                    if (g.residual) c += g.residual[(m_strip + r) * g.ldc + n];
                    if (g.relu) c = fmaxf(c, 0.0f);
                    __builtin_nontemporal_store(c, g.C + (m_strip + r) * g.ldc + n);
                    mx = fmaxf(mx, fabsf(c));
                }
            }
        }
    }
    if (FOLD && g.absmax_bits) fold_absmax(g.absmax_bits, mx);
    return mx;
}

}  // namespace dybit
#endif
