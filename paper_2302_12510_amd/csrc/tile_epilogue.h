// Epilogue shared by the tiled matrix-product kernels: C = acc * (sA sW) (+ bias) (+ residual) (ReLU),
// sW the scale of the weight tensor or of the output column's weight row (g.w_per_channel), the residual
// (shortcut) an fp32 tensor or, in the write-back build, a tensor of DyBit codes with a scale of its own,
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

// Shortcut tensor given as DyBit codes (Sec. III-B: activations live in memory as codes): the value added
// is fl(s_r * value(code)), the number dybit_dequantize writes.  RES_TABLE (4- and 6-bit codes): lane i of a
// register holds that number for code i and a value is fetched with one cross-lane read.  RES_ARITH (8-bit
// codes): the decoder identity of dybit_codec.h in fp32 -- with n = 2^m - magnitude,
// value * 2^-126 = bitcast(((127 + m) << 23) - bits(float(n))) over the whole range (a subnormal below 1).
enum { RES_NONE = 0, RES_F32 = 1, RES_TABLE = 2, RES_ARITH = 3 };

struct ResCodes {
    uint32_t m, mag_mask, two_m, recip_sub, sign_shift;   // magnitude bits, 2^m - 1, 2^m, (127 + m) << 23, 31 - m
    float s;                                              // the shortcut tensor's scale
    uint32_t code_mask;                                   // 2^bits - 1
    uint32_t table;                                       // RES_TABLE: bits of fl(s * value(lane))
};

__device__ __forceinline__ float res_value(uint32_t code, const ResCodes &r)
{
    const float n = (float)(r.two_m - (code & r.mag_mask));
    const float v = __uint_as_float(r.recip_sub - __float_as_uint(n)) * __uint_as_float(0x7E800000u);   // * 2^126: exact
    return __uint_as_float(__float_as_uint(v * r.s) ^ ((code << r.sign_shift) & 0x80000000u));
}

__device__ __forceinline__ ResCodes make_res_codes(const GemmArgs &g, int lane)
{
    ResCodes r;
    const int m = g.res_signed ? g.res_bits - 1 : g.res_bits;
    r.m = (uint32_t)m;
    r.mag_mask = (1u << m) - 1u;
    r.two_m = 1u << m;
    r.recip_sub = (uint32_t)(127 + m) << 23;
    r.sign_shift = (uint32_t)(31 - m);                    // unsigned format: bit m of a code is never set
    r.s = *g.res_scale;
    r.code_mask = (1u << g.res_bits) - 1u;
    r.table = __float_as_uint(res_value((uint32_t)lane & r.code_mask, r));
    return r;
}

// The same strip with the write-back encoder (requant.h): per 32 x 32 block, three phases over the
// lane's values (eight at a time) so that the instruction streams of the values interleave and the only branch is
// one per block -- (1) result, optional fp32 store, rounded real-valued code; (2) only if some
// lane's value sits within 2^-G of a decision point: the exact decision for those;
// (3) sign, packing across lanes, store of the packed words through a descriptor of their own.
// A NULL fp32 output becomes an empty descriptor whose stores the hardware drops.
template <int CB, int RES, int BITS, int ACC_EXP>
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
    constexpr bool HAS_RES = RES != RES_NONE, RES_CODES = RES == RES_TABLE || RES == RES_ARITH;
    const uint32_t rrow = RES_CODES ? (uint32_t)g.res_row_bytes : ldc4;       // bytes from a shortcut row to the next
    const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(
        RES_CODES ? const_cast<uint8_t *>(g.res_codes + m_strip * g.res_row_bytes)
                  : reinterpret_cast<uint8_t *>(const_cast<float *>(RES == RES_F32 ? g.residual + m_strip * g.ldc : g.a_scale)),
        0, HAS_RES ? (int)((uint32_t)rows * rrow) : 0, 0x00020000);
    ResCodes rc{};
    if (RES_CODES) rc = make_res_codes(g, lane);
    const bool res_six = RES == RES_TABLE && g.res_bits == 6;               // uniform: a 6-bit code may straddle two bytes
    const uint32_t qrow = (uint32_t)g.q_row_bytes;
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(g.q_out + m_strip * g.q_row_bytes, 0,
                                                                        (int)((uint32_t)rows * qrow), 0x00020000);
    const Requant rqp = make_requant(g.q_scale, BITS, g.q_signed);
    if (!rqp.ok && m_strip == 0 && n0 == 0 && lane == 0) *g.async_error = DYBIT_ERR_BAD_SCALE;   // no codes, flag the call
    constexpr int GV = 8;
    const bool track = g.absmax_bits != nullptr;
    // ReLU as a maximum with a uniform floor (no select per value).  Without ReLU the floor is NaN:
    // the maximum of a number and NaN is the number, and a NaN result stays NaN (and becomes code 0)
    uint32_t floor_bits = (uint32_t)__builtin_amdgcn_readfirstlane(g.relu ? 0 : 0x7fc00000);
    asm volatile("" : "+s"(floor_bits));                               // opaque: else the maximum becomes a maximum and a select per value
    const float relu_floor = __uint_as_float(floor_bits);
    float mx = 0.0f;
    constexpr bool PREFETCH = HAS_RES && CB <= 4;
    // fp32 shortcut: the value's bits; codes: the byte that holds the code (6-bit: that byte and the next one in
    // the upper half), shifted and decoded when the value is used
    uint32_t res2[2][GV];
    uint32_t roff = 0;                                                  // walks the shortcut's rows like `off` walks C's
    // position of the lane's code inside its byte: the same in every column block (32 codes are whole bytes)
    const uint32_t rshift = RES_CODES ? (uint32_t)(((n0 + col) * g.res_bits) & 7) : 0u;
    auto load_shortcut = [&](int first_v, uint32_t (&r)[GV]) {
#pragma unroll
        for (int u = 0; u < GV; ++u) {
            if (RES_CODES) {
                r[u] = __builtin_amdgcn_raw_buffer_load_b8(rres, roff, 0, 0);
                if (res_six) r[u] |= (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(rres, roff + 1u, 0, 0) << 8;
            } else {
                r[u] = __builtin_amdgcn_raw_buffer_load_b32(rres, roff, 0, 0);
            }
            roff += ((first_v + u) & 3) == 3 ? 5u * rrow : rrow;
        }
    };
    auto shortcut_offset = [&](int64_t n, bool n_ok) {                  // byte offset of column n in the lane's first row
        const uint32_t first = RES_CODES ? ((uint32_t)n * (uint32_t)g.res_bits) >> 3 : (uint32_t)n * 4u;
        return (n_ok ? first : 0x80000000u) + (uint32_t)(4 * kq) * rrow;
    };
    auto shortcut_value = [&](uint32_t raw) -> float {
        if (RES == RES_F32) return __uint_as_float(raw);
        const uint32_t code = (raw >> rshift) & rc.code_mask;
        if (RES == RES_TABLE) return __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute((int)(code << 2), (int)rc.table));
        return res_value(code, rc);
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
        if (HAS_RES && (j == 0 || !PREFETCH)) { roff = shortcut_offset(n, n_ok); if (PREFETCH) load_shortcut(0, res2[0]); }
#pragma unroll
        for (int h = 0; h < 16; h += GV) {                                   // GV values at a time: fewer live registers
            // the shortcut values of the next group are requested before this group is stored (see
            // store_strip) where the kernel has registers for them; else they are loaded here
            const int grp = (j * 16 + h) / GV;
            uint32_t (&res)[GV] = res2[PREFETCH ? (grp & 1) : 0];
            if (HAS_RES && !PREFETCH) load_shortcut(h, res);
            if (PREFETCH) {
                if (h + GV < 16) {
                    load_shortcut(h + GV, res2[(grp + 1) & 1]);
                } else if (j + 1 < CB) {
                    const int64_t n1 = n0 + (j + 1) * 32 + col;
                    roff = shortcut_offset(n1, n1 < g.N);
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
                if (HAS_RES) c[u] += shortcut_value(res[u]);
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
    if (WB) {                                                       // the host has checked ldc, N and the formats
#define DYBIT_WB_STRIP(RES_) \
        mx = g.q_bits == 4 ? store_strip_wb<CB, RES_, 4, ACC_EXP>(g, acc, m_strip, n0, rows, alpha) \
           : g.q_bits == 8 ? store_strip_wb<CB, RES_, 8, ACC_EXP>(g, acc, m_strip, n0, rows, alpha) \
                           : store_strip_wb<CB, RES_, 6, ACC_EXP>(g, acc, m_strip, n0, rows, alpha)
        if (g.residual) { DYBIT_WB_STRIP(RES_F32); }
        else if (!g.res_codes) { DYBIT_WB_STRIP(RES_NONE); }
        else if (g.res_bits == 8) { DYBIT_WB_STRIP(RES_ARITH); }
        else { DYBIT_WB_STRIP(RES_TABLE); }
#undef DYBIT_WB_STRIP
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
