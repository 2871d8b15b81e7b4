// DyBit per-tensor scale, quantize (encoder) and dequantize (decoder) kernels for gfx950,
// with their C-ABI entry points.  These passes are bound by HBM bandwidth: every load and
// store is a full-width coalesced vector access and each element is touched once.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "dybit_device.h"
#include "dybit_host.h"

namespace dybit {

__device__ int g_async_error = 0;

constexpr int kThreads = 256;
// Tuning knobs of the quantize pass (swept on the device, from 2^20 to 2^28 elements: four 128-bit loads
// in flight per lane and a grid that is not capped below about 128 workgroups per compute unit run
// closest to the HBM rate -- 2 to 9 % faster than eight loads; tensors of under 2^23 elements (most
// activation tensors of the networks) have too few workgroups then and take two loads per lane).
#ifndef DYBIT_QUANT_UNROLL
#define DYBIT_QUANT_UNROLL 4
#endif
#define DYBIT_QUANT_UNROLL_SMALL 2
constexpr size_t kQuantSmall = (size_t)1 << 21;     // in groups of four elements
#ifndef DYBIT_QUANT_BLOCKS_PER_CU
#define DYBIT_QUANT_BLOCKS_PER_CU 128
#endif
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// absmax -> scale
// ---------------------------------------------------------------------------
// Non-negative floats order like their bit patterns, so the running maximum is kept with an
// integer atomicMax directly in the output word; NaNs are dropped by fmaxf before that.
__global__ void absmax_init_kernel(float *scale_out) { *scale_out = 0.0f; }

__global__ __launch_bounds__(kThreads) void absmax_kernel(const float *__restrict__ x, size_t n,
                                                          float *scale_out)
{
    // A workgroup reads contiguous chunks of 4 x kThreads 128-bit words (16 KiB), four loads in flight per
    // lane.  (A lane whose four loads are a whole grid apart -- a large power of two -- keeps hitting
    // the same memory channels: that form measured 5.4 TB/s against 7.0 TB/s for this one.)
    const size_t n4 = n >> 2;
    const f32x4 *x4 = reinterpret_cast<const f32x4 *>(x);
    float mx = 0.0f;
    constexpr size_t per_block = (size_t)kThreads * 4;
    for (size_t base = (size_t)blockIdx.x * per_block; base < n4; base += (size_t)gridDim.x * per_block) {
        const size_t i = base + threadIdx.x;
        f32x4 v[4];
        if (base + per_block <= n4) {                                  // uniform: a whole chunk
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(x4 + i + u * kThreads);
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = (i + u * kThreads < n4) ? x4[i + u * kThreads] : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            mx = fmaxf(mx, fmaxf(fmaxf(fabsf(v[u].x), fabsf(v[u].y)), fmaxf(fabsf(v[u].z), fabsf(v[u].w))));
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) mx = fmaxf(mx, fabsf(x[(n4 << 2) + threadIdx.x]));
    // At most one atomic per workgroup, and only when it would raise the word: atomics on a single address
    // serialise in L2 (about 10 ns each).  A stale read can only cause a needless atomic.
    __shared__ float wave_max[kThreads / 64];
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) mx = fmaxf(mx, wave_max[w]);
        unsigned int *word = reinterpret_cast<unsigned int *>(scale_out);
        const unsigned int bits = __float_as_uint(mx);
        if (bits > __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(word, bits);
    }
}

__global__ void absmax_to_scale_kernel(const float *absmax, float *scale_out, float inv_vmax)
{
    const float mx = *absmax;
    *scale_out = (mx == 0.0f) ? 1.0f : mx * inv_vmax;   // division by 2^(m-1): exact
}

__global__ void absmax_finish_kernel(float *scale_out, float inv_vmax)
{
    const float mx = *scale_out;
    *scale_out = (mx == 0.0f) ? 1.0f : mx * inv_vmax;   // division by 2^(m-1): exact
}

// ---------------------------------------------------------------------------
// quantize
// ---------------------------------------------------------------------------
// The result must be the code nearest to x in exact arithmetic, but x / s cannot be formed
// exactly in float.  Two paths:
//
//  fast  q = min(|x| * fl(1/s), vmax) is within 2^-23 (relative) of the true quotient t.  The
//        "real-valued code" c(t) -- t * 2^(m-1) below 1, then the inverse of magnitude_value -- is
//        piecewise linear, continuous, and the decision points are exactly its half-integers.
//        One expression yields n = 2^m - c(q) over the whole range: with q' = q * 2^-126,
//        n = bitcast(((127 + m) << 23) - bits(q')).  For q >= 1 that is the decoder's identity read
//        backwards; for q < 1, q' is a subnormal float whose bits are q * 2^23, linear in q, and the
//        difference lands in the top binade [2^(m-1), 2^m] at 2^m - q 2^(m-1).  n is rounded to
//        G fractional bits with one magic-number addition; unless those bits read exactly
//        one half, q and t are on the same side of every decision point and the code is the
//        integer part rounded half up.  Error budget: |c(q) - c(t)| <= 1.5 * 2^(m-24) < 2^-(G+1).
//        A NaN becomes q = 0 (v_med3_f32 returns the minimum of its other operands for a NaN).
//  exact when the G bits read one half (probability 2^-G), and for scales so
//        extreme that 1/s or the product could leave the normal range: the side of the
//        decision point is the sign of fma(-s, mid, |x|), which is exact; zero is a tie and
//        goes to the even code.
template <int M>
struct QConst {
    static constexpr int G = 13;                                       // 1.5 * 2^(M-24) < 2^-(G+1) for M <= 8; 2^M + magic stays in magic's binade
    static constexpr uint32_t kRecip = (uint32_t)(254 + M - 1) << 23;  // see magnitude_value
    static constexpr uint32_t kRecipSub = (uint32_t)(127 + M) << 23;   // the same constant for an argument scaled by 2^-126
    static constexpr uint32_t kMagic = ((uint32_t)(127 + 23 - G) << 23) | 0x400000u;  // 1.5 * 2^(23-G)
    static constexpr uint32_t kRound = kMagic + (1u << (G - 1));
    static constexpr uint32_t kTop = (1u << M) - 1;
};

// Decision point between magnitude codes j and j+1, as a float (exact: <= 9 significant bits).
template <int M>
__device__ __forceinline__ float midpoint_value(uint32_t j)
{
    const float h = (float)j + 0.5f;
    if (j < (1u << (M - 1)))                       // lower neighbour is a pure fraction; so is the
        return h * __uint_as_float((uint32_t)(127 - (M - 1)) << 23);   // grid up to and including 1.0
    return __uint_as_float(QConst<M>::kRecip - __float_as_uint((float)(1u << M) - h));
}

// Exact magnitude code of |x| / s.  ax = |x| (not NaN), s a finite normal positive float.
template <int M>
__device__ __noinline__ uint32_t magnitude_exact(float ax, float s)
{
    // Scale both by the same power of two so that s2 is in [1, 2): the fma below then cannot
    // lose its sign to underflow for any |x| near a decision point, and multiplying by a power
    // of two is exact (an overflow to Inf or an underflow of a negligible |x| keeps the order).
    const uint32_t sb = __float_as_uint(s);
    const float p = __uint_as_float((254u - (sb >> 23)) << 23);
    const float s2 = s * p, ax2 = ax * p;
    float t = fminf(ax2 / s2, (float)(1u << (M - 1)));
    float c = (t < 1.0f) ? t * (float)(1u << (M - 1))
                         : (float)(1u << M) - __uint_as_float(QConst<M>::kRecip - __float_as_uint(t));
    uint32_t j = min((uint32_t)c, QConst<M>::kTop);
    // j is within one of the answer; settle it with exact comparisons.
    while (j < QConst<M>::kTop) {
        const float r = fmaf(-s2, midpoint_value<M>(j), ax2);            // sign(|x| - s * mid_j), exact
        if (r > 0.0f || (r == 0.0f && (j & 1u))) ++j; else break;
    }
    while (j > 0) {
        const float r = fmaf(-s2, midpoint_value<M>(j - 1), ax2);
        if (r < 0.0f || (r == 0.0f && (j & 1u))) --j; else break;
    }
    return j;
}

template <int BITS, bool SIGNED>
__device__ __forceinline__ uint32_t quantize_exact(float x, float s)
{
    constexpr int M = SIGNED ? BITS - 1 : BITS;
    if (x != x) return 0u;
    const bool neg = __float_as_uint(x) >> 31;
    if (!SIGNED && neg) return 0u;
    const uint32_t j = magnitude_exact<M>(fabsf(x), s);
    return (SIGNED && neg && j) ? (j | (1u << M)) : j;
}

// Fast path for one element: kRound minus the rounded n, i.e. the magnitude code in bits G .. G+M-1
// (rounded half up) above G fraction bits that are all zero exactly when the exact path must decide.
template <int BITS, bool SIGNED>
__device__ __forceinline__ uint32_t quantize_fast_raw(float x, float rinv)
{
    constexpr int M = SIGNED ? BITS - 1 : BITS;
    using K = QConst<M>;
    const float vmax = (float)(1u << (M - 1));
    const float t = x * rinv;
    const float q = SIGNED ? __builtin_amdgcn_fmed3f(fabsf(t), 0.0f, vmax) : __builtin_amdgcn_fmed3f(t, 0.0f, vmax);   // NaN -> 0
    const float qs = q * __uint_as_float(1u << 23);                      // q * 2^-126
    const float nf = __uint_as_float(K::kRecipSub - __float_as_uint(qs));   // 2^m - c (-2^m should the median of -0, 0, vmax be -0)
    return K::kRound - __float_as_uint(fabsf(nf) + __uint_as_float(K::kMagic));
}

// One element: the code (sign included, possibly a negative zero); sets `redo` when the exact path must decide.
template <int BITS, bool SIGNED>
__device__ __forceinline__ uint32_t quantize_fast(float x, float rinv, bool &redo)
{
    constexpr int M = SIGNED ? BITS - 1 : BITS;
    using K = QConst<M>;
    const uint32_t r = quantize_fast_raw<BITS, SIGNED>(x, rinv);
    redo = (r << (32 - K::G)) == 0u;
    uint32_t code = (r >> K::G) & K::kTop;
    if (SIGNED) code |= (__float_as_uint(x) >> (31 - M)) & (1u << M);
    return code;
}

// Four elements: their codes packed into fields of BITS bits (negative zeros cleared); sets `redo`
// when the exact path must decide one of them.
template <int BITS>
__device__ __forceinline__ uint32_t clear_negative_zero(uint32_t w);
template <int BITS, bool SIGNED>
__device__ __forceinline__ uint32_t quantize_fast4(const float (&e)[4], float rinv, bool &redo)
{
    constexpr int M = SIGNED ? BITS - 1 : BITS;
    using K = QConst<M>;
    uint32_t r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) r[k] = quantize_fast_raw<BITS, SIGNED>(e[k], rinv);
    // the smallest of the four fraction fields (moved to the top of the word) is zero when one of them is
    redo = min(min(r[0] << (32 - K::G), r[1] << (32 - K::G)), min(r[2] << (32 - K::G), r[3] << (32 - K::G))) == 0u;
    uint32_t w = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) w |= ((r[k] >> K::G) & K::kTop) << (k * BITS);
    if (SIGNED) {
#pragma unroll
        for (int k = 0; k < 4; ++k) w |= (__float_as_uint(e[k]) >> (31 - M - k * BITS)) & (1u << (M + k * BITS));
        w = clear_negative_zero<BITS>(w);
    }
    return w;
}

// Clears the sign bit of every field whose magnitude is zero (four fields of BITS bits in a word).
template <int BITS>
__device__ __forceinline__ uint32_t clear_negative_zero(uint32_t w)
{
    constexpr uint32_t ones = 1u | (1u << BITS) | (1u << (2 * BITS)) | (1u << (3 * BITS));
    constexpr uint32_t sign = ones << (BITS - 1);
    constexpr uint32_t magm = sign - ones;
    const uint32_t t = w & magm;
    return t | (w & (t + magm) & sign);
}

struct ScaleInfo {
    float s, rinv;
    bool ok, all_exact;
};

// inv_vmax > 0: *scale holds max|x| instead of the scale; the scale is max|x| * inv_vmax (1.0 for a
// maximum of 0), exactly what dybit_scale_from_absmax computes, and the first thread of the grid
// writes it to *scale_out for the kernels that follow.
__device__ __forceinline__ ScaleInfo load_scale(const float *scale, float inv_vmax = 0.0f, float *scale_out = nullptr)
{
    ScaleInfo si;
    si.s = *scale;
    if (inv_vmax > 0.0f) {
        si.s = (si.s == 0.0f) ? 1.0f : si.s * inv_vmax;
        if (blockIdx.x == 0 && threadIdx.x == 0) *scale_out = si.s;
    }
    const uint32_t e = (__float_as_uint(si.s) >> 23) & 0xffu;
    si.ok = (si.s > 0.0f) && e != 0u && e != 255u;                      // finite, normal, positive
    si.all_exact = e < 27u || e > 227u;                                 // outside [2^-100, 2^100]
    si.rinv = 1.0f / si.s;
    return si;
}

// 4 consecutive elements per lane per load (coalesced float4), UNROLL loads in flight; a workgroup works
// on contiguous chunks of UNROLL x kThreads loads.  Whole chunks run without bounds checks.
// Output per load: 4*BITS bits, stored as one 8/16/32-bit word.  BITS in {2, 4, 8}.
template <int BITS, bool SIGNED, int UNROLL>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const float *__restrict__ x, size_t n4,
                                                            const float *__restrict__ scale,
                                                            uint8_t *__restrict__ out, float inv_vmax, float *scale_out, int *err)
{
    using word_t = typename std::conditional<BITS == 8, uint32_t,
                   typename std::conditional<BITS == 4, uint16_t, uint8_t>::type>::type;
    const ScaleInfo si = load_scale(scale, inv_vmax, scale_out);
    if (!si.ok) {
        if (blockIdx.x == 0 && threadIdx.x == 0) *err = DYBIT_ERR_BAD_SCALE;
        return;
    }
    const f32x4 *x4 = reinterpret_cast<const f32x4 *>(x);
    word_t *o = reinterpret_cast<word_t *>(out);
    auto encode = [&](const f32x4 v) -> uint32_t {
        const float e[4] = {v.x, v.y, v.z, v.w};
        bool redo;
        uint32_t w = quantize_fast4<BITS, SIGNED>(e, si.rinv, redo);
        if (redo | si.all_exact) {
            w = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) w |= quantize_exact<BITS, SIGNED>(e[k], si.s) << (k * BITS);
        }
        return w;
    };
    constexpr size_t per_block = (size_t)kThreads * UNROLL;
    for (size_t base = (size_t)blockIdx.x * per_block; base < n4; base += (size_t)gridDim.x * per_block) {
        const size_t i = base + threadIdx.x;
        f32x4 v[UNROLL];
        if (base + per_block <= n4) {                                  // uniform: a whole chunk
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(x4 + i + u * kThreads);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) __builtin_nontemporal_store((word_t)encode(v[u]), o + i + u * kThreads);
        } else {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                v[u] = (i + u * kThreads < n4) ? __builtin_nontemporal_load(x4 + i + u * kThreads) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t w = encode(v[u]);
                if (i + u * kThreads < n4) __builtin_nontemporal_store((word_t)w, o + i + u * kThreads);
            }
        }
    }
}

// 6-bit: like the kernel above, each lane takes a coalesced float4 and produces four codes (24 bits);
// four neighbouring lanes' 96 bits are three words.  Lane k of a group of four (k < 3) fetches its
// right neighbour's 24 bits and stores word k = (own >> 8k) | (neighbour << (24 - 8k)), so loads and
// stores are both fully coalesced.  n4 must be a multiple of 4 (whole groups of 16 elements).
template <bool SIGNED, int UNROLL>
__global__ __launch_bounds__(kThreads) void quantize6_kernel(const float *__restrict__ x, size_t n4,
                                                             const float *__restrict__ scale,
                                                             uint8_t *__restrict__ out, float inv_vmax, float *scale_out, int *err)
{
    const ScaleInfo si = load_scale(scale, inv_vmax, scale_out);
    if (!si.ok) {
        if (blockIdx.x == 0 && threadIdx.x == 0) *err = DYBIT_ERR_BAD_SCALE;
        return;
    }
    const f32x4 *x4 = reinterpret_cast<const f32x4 *>(x);
    uint32_t *o = reinterpret_cast<uint32_t *>(out);
    const int k = threadIdx.x & 3;
    const size_t per_block = (size_t)kThreads * UNROLL;
    for (size_t base = (size_t)blockIdx.x * per_block; base < n4; base += (size_t)gridDim.x * per_block) {
        f32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const size_t i = base + (size_t)u * kThreads + threadIdx.x;
            v[u] = (i < n4) ? __builtin_nontemporal_load(x4 + i) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const size_t i = base + (size_t)u * kThreads + threadIdx.x;
            const float e[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
            bool redo;
            uint32_t own = quantize_fast4<6, SIGNED>(e, si.rinv, redo);   // four 6-bit fields
            if (redo | si.all_exact) {
                own = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) own |= quantize_exact<6, SIGNED>(e[j], si.s) << (6 * j);
            }
            const uint32_t right = __shfl_down(own, 1, 64);              // every lane takes part; lane 3 of a group ignores it
            const uint32_t w = (own >> (8 * k)) | (right << (24 - 8 * k));
            if (k < 3 && i < n4) __builtin_nontemporal_store(w, o + (i >> 2) * 3 + k);
        }
    }
}

// quantize followed by dequantize without the codes ever reaching memory (the forward of the
// quantization-aware training step, Sec. III-C): y = s * value(code of x), bit for bit what
// dybit_dequantize returns for dybit_quantize's codes.  8 bytes per element.
template <int BITS, bool SIGNED>
__device__ __forceinline__ float code_to_value(uint32_t code, float s)
{
    return s * code_value(code, BITS, SIGNED);                           // the expression of the dequantize table
}

template <int BITS, bool SIGNED, int UNROLL>
__global__ __launch_bounds__(kThreads) void fake_quant_kernel(const float *__restrict__ x, size_t n,
                                                              const float *__restrict__ scale, float *__restrict__ y, int *err)
{
    const ScaleInfo si = load_scale(scale);
    if (!si.ok) {
        if (blockIdx.x == 0 && threadIdx.x == 0) *err = DYBIT_ERR_BAD_SCALE;
        return;
    }
    const size_t n4 = n >> 2;
    const f32x4 *x4 = reinterpret_cast<const f32x4 *>(x);
    f32x4 *y4 = reinterpret_cast<f32x4 *>(y);
    const size_t per_block = (size_t)kThreads * UNROLL;
    for (size_t base = (size_t)blockIdx.x * per_block; base < n4; base += (size_t)gridDim.x * per_block) {
        f32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const size_t i = base + (size_t)u * kThreads + threadIdx.x;
            v[u] = (i < n4) ? __builtin_nontemporal_load(x4 + i) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const size_t i = base + (size_t)u * kThreads + threadIdx.x;
            const float e[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
            uint32_t c[4];
            bool any_redo = si.all_exact;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                bool redo;
                c[k] = quantize_fast<BITS, SIGNED>(e[k], si.rinv, redo);
                any_redo |= redo;
            }
            if (any_redo) {
#pragma unroll
                for (int k = 0; k < 4; ++k) c[k] = quantize_exact<BITS, SIGNED>(e[k], si.s);
            }
            const f32x4 out = {code_to_value<BITS, SIGNED>(c[0], si.s), code_to_value<BITS, SIGNED>(c[1], si.s),
                               code_to_value<BITS, SIGNED>(c[2], si.s), code_to_value<BITS, SIGNED>(c[3], si.s)};
            if (i < n4) __builtin_nontemporal_store(out, y4 + i);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {                      // remainder: exact path
        const size_t j = (n4 << 2) + threadIdx.x;
        y[j] = code_to_value<BITS, SIGNED>(quantize_exact<BITS, SIGNED>(x[j], si.s), si.s);
    }
}

// Remainder: one thread per group of 4 elements starting at element `first`; exact path, byte stores.
template <int BITS, bool SIGNED>
__global__ void quantize_tail_kernel(const float *__restrict__ x, size_t first, size_t n,
                                     const float *__restrict__ scale, uint8_t *__restrict__ out, float inv_vmax, float *scale_out,
                                     int *err)
{
    const ScaleInfo si = load_scale(scale, inv_vmax, scale_out);
    if (!si.ok) {
        if (blockIdx.x == 0 && threadIdx.x == 0) *err = DYBIT_ERR_BAD_SCALE;
        return;
    }
    const size_t e0 = first + 4 * ((size_t)blockIdx.x * blockDim.x + threadIdx.x);
    if (e0 >= n) return;
    uint32_t w = 0;
    int cnt = 0;
    for (int k = 0; k < 4 && e0 + k < n; ++k, ++cnt) w |= quantize_exact<BITS, SIGNED>(x[e0 + k], si.s) << (k * BITS);
    const size_t byte0 = e0 * BITS / 8;                                  // e0 is a multiple of 4
    const int nbytes = (cnt * BITS + 7) / 8;
    for (int b = 0; b < nbytes; ++b) out[byte0 + b] = (uint8_t)(w >> (8 * b));
}

// Row-wise (per-output-channel) max-abs scale and codes of a weight matrix: one workgroup per row,
// first the row's maximum, then the exact encoder on every element.  Weight tensors are small and
// are encoded once, so this kernel is written for clarity: a thread produces whole bytes (8-bit: one
// code, 4-bit: two, 2-bit: four, 6-bit: four codes in three bytes).
template <int BITS, bool SIGNED>
__global__ __launch_bounds__(kThreads) void quantize_rows_kernel(const float *__restrict__ x, int64_t cols, float inv_vmax,
                                                                 float *__restrict__ scales, uint8_t *__restrict__ out, int *err)
{
    constexpr int EPG = BITS == 8 ? 1 : BITS == 4 ? 2 : 4;             // elements per group of whole bytes
    constexpr int BPG = BITS == 6 ? 3 : 1;
    const float *row = x + (int64_t)blockIdx.x * cols;
    uint8_t *orow = out + (int64_t)blockIdx.x * (cols * BITS / 8);
    float mx = 0.0f;
    for (int64_t i = threadIdx.x; i < cols; i += kThreads) mx = fmaxf(mx, fabsf(row[i]));
    __shared__ float wave_max[kThreads / 64];
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
    const float s = (mx == 0.0f) ? 1.0f : mx * inv_vmax;               // as dybit_absmax_scale
    if (threadIdx.x == 0) scales[blockIdx.x] = s;
    const uint32_t e = (__float_as_uint(s) >> 23) & 0xffu;
    if (!(s > 0.0f) || e == 0u || e == 255u) {                         // an infinite or subnormal maximum: no codes
        if (threadIdx.x == 0) *err = DYBIT_ERR_BAD_SCALE;
        return;
    }
    for (int64_t gi = threadIdx.x; gi < cols / EPG; gi += kThreads) {
        uint32_t w = 0;
#pragma unroll
        for (int k = 0; k < EPG; ++k) w |= quantize_exact<BITS, SIGNED>(row[gi * EPG + k], s) << (k * BITS);
#pragma unroll
        for (int b = 0; b < BPG; ++b) orow[gi * BPG + b] = (uint8_t)(w >> (8 * b));
    }
}

// Column-wise (per-channel, channel innermost) max-abs scales of a matrix [rows][cols]: a workgroup owns
// 64 neighbouring columns, four row lanes each, so that the loads of a wave are contiguous.
__global__ __launch_bounds__(kThreads) void col_scale_kernel(const float *__restrict__ x, int64_t rows, int64_t cols, float inv_vmax,
                                                             float *__restrict__ scales)
{
    const int c_local = threadIdx.x & 63, r_lane = threadIdx.x >> 6;
    const int64_t c = (int64_t)blockIdx.x * 64 + c_local;
    float mx = 0.0f;
    if (c < cols)
        for (int64_t r = r_lane; r < rows; r += kThreads / 64) mx = fmaxf(mx, fabsf(x[r * cols + c]));
    __shared__ float part[kThreads / 64][64];
    part[r_lane][c_local] = mx;
    __syncthreads();
    if (r_lane == 0 && c < cols) {
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) mx = fmaxf(mx, part[w][c_local]);
        scales[c] = (mx == 0.0f) ? 1.0f : mx * inv_vmax;              // as dybit_absmax_scale
    }
}

// Codes of a matrix [rows][cols] under one scale per column: a thread produces whole bytes (see
// quantize_rows_kernel), every element with the exact encoder under its own column's scale.
template <int BITS, bool SIGNED>
__global__ __launch_bounds__(kThreads) void quantize_cols_kernel(const float *__restrict__ x, int64_t cols, int64_t groups,
                                                                 const float *__restrict__ scales, uint8_t *__restrict__ out, int *err)
{
    constexpr int EPG = BITS == 8 ? 1 : BITS == 4 ? 2 : 4;             // elements per group of whole bytes
    constexpr int BPG = BITS == 6 ? 3 : 1;
    const int64_t gi = (int64_t)blockIdx.x * kThreads + threadIdx.x;   // cols is a multiple of EPG: a group stays inside a row
    if (gi >= groups) return;
    uint32_t w = 0;
    bool bad = false;
#pragma unroll
    for (int k = 0; k < EPG; ++k) {
        const int64_t i = gi * EPG + k;
        const float s = scales[i % cols];
        const uint32_t e = (__float_as_uint(s) >> 23) & 0xffu;
        const bool ok = s > 0.0f && e != 0u && e != 255u;              // an infinite or subnormal maximum: code 0
        bad |= !ok;
        w |= (ok ? quantize_exact<BITS, SIGNED>(x[i], s) : 0u) << (k * BITS);
    }
#pragma unroll
    for (int b = 0; b < BPG; ++b) out[gi * BPG + b] = (uint8_t)(w >> (8 * b));
    if (bad) *err = DYBIT_ERR_BAD_SCALE;
}

// Encoder for a matrix whose rows are padded with zero codes on the way: row r of x holds `cols` floats, row r of
// the output cols_padded codes (a few-channel image whose pixels must end on a byte or word boundary, e.g. 3 -> 4
// channels).  One thread per group of four output codes (bits / 2 bytes), every element through the exact
// encoder; consecutive threads read and write consecutive memory.
template <int BITS, bool SIGNED>
__global__ __launch_bounds__(kThreads) void quantize_pad_kernel(const float *__restrict__ x, int cols, int groups_per_row, int64_t groups,
                                                                const float *__restrict__ scale, uint8_t *__restrict__ out, int *err)
{
    const ScaleInfo si = load_scale(scale);
    if (!si.ok) {                                                      // as dybit_quantize: nothing is written
        if (blockIdx.x == 0 && threadIdx.x == 0) *err = DYBIT_ERR_BAD_SCALE;
        return;
    }
    for (int64_t gi = (int64_t)blockIdx.x * kThreads + threadIdx.x; gi < groups; gi += (int64_t)gridDim.x * kThreads) {
        const int64_t row = gi / groups_per_row;
        const int c0 = (int)(gi - row * groups_per_row) * 4;
        const float *src = x + row * cols;
        float e[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) e[k] = c0 + k < cols ? src[c0 + k] : 0.0f;   // the padding: value 0, code 0
        bool redo;
        uint32_t w = quantize_fast4<BITS, SIGNED>(e, si.rinv, redo);
        if (redo | si.all_exact) {
            w = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) w |= quantize_exact<BITS, SIGNED>(e[k], si.s) << (k * BITS);
        }
        uint8_t *dst = out + gi * (BITS / 2);
        if constexpr (BITS == 8) *reinterpret_cast<uint32_t *>(dst) = w;       // groups are whole, aligned words / halves
        else if constexpr (BITS == 4) *reinterpret_cast<uint16_t *>(dst) = (uint16_t)w;
        else {
#pragma unroll
            for (int b = 0; b < BITS / 2; ++b) dst[b] = (uint8_t)(w >> (8 * b));
        }
    }
}

// Straight-through gradient of the quantize-then-decode operator: the incoming gradient where x lies
// inside [lo, hi] (bounds included), zero elsewhere and for NaN.  12 bytes per element.
__global__ __launch_bounds__(kThreads) void fake_quant_bwd_kernel(const float *__restrict__ x, const float *__restrict__ grad, size_t n,
                                                                  const float *__restrict__ scale, float vmax, int is_signed,
                                                                  float *__restrict__ out, int *err)
{
    const float s = *scale;
    if (!(s > 0.0f) || ((__float_as_uint(s) >> 23) & 0xffu) == 255u) {
        if (blockIdx.x == 0 && threadIdx.x == 0) *err = DYBIT_ERR_BAD_SCALE;
        return;
    }
    // s * 2^(m-1) is exact; should it overflow, every finite x is inside and +Inf is not
    const float hi = fminf(s * vmax, __uint_as_float(0x7f7fffffu)), lo = is_signed ? -hi : 0.0f;
    const size_t n4 = n >> 2;
    const f32x4 *x4 = reinterpret_cast<const f32x4 *>(x), *g4 = reinterpret_cast<const f32x4 *>(grad);
    f32x4 *o4 = reinterpret_cast<f32x4 *>(out);
    auto mask = [&](f32x4 xv, f32x4 gv) {
        f32x4 r;
#pragma unroll
        for (int k = 0; k < 4; ++k) r[k] = (xv[k] >= lo && xv[k] <= hi) ? gv[k] : 0.0f;
        return r;
    };
    constexpr size_t per_block = (size_t)kThreads * 2;
    for (size_t base = (size_t)blockIdx.x * per_block; base < n4; base += (size_t)gridDim.x * per_block) {
        const size_t i = base + threadIdx.x;
        if (base + per_block <= n4) {                                  // uniform: a whole chunk, four loads in flight
            const f32x4 a0 = __builtin_nontemporal_load(x4 + i), a1 = __builtin_nontemporal_load(x4 + i + kThreads);
            const f32x4 b0 = __builtin_nontemporal_load(g4 + i), b1 = __builtin_nontemporal_load(g4 + i + kThreads);
            __builtin_nontemporal_store(mask(a0, b0), o4 + i);
            __builtin_nontemporal_store(mask(a1, b1), o4 + i + kThreads);
        } else {
            for (int u = 0; u < 2; ++u)
                if (i + u * kThreads < n4) o4[i + u * kThreads] = mask(x4[i + u * kThreads], g4[i + u * kThreads]);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const size_t j = (n4 << 2) + threadIdx.x;
        out[j] = (x[j] >= lo && x[j] <= hi) ? grad[j] : 0.0f;
    }
}

// ---------------------------------------------------------------------------
// dequantize
// ---------------------------------------------------------------------------
// Table of s * value(code) in LDS (one multiply per entry, as the definition says).  A lane expands one
// group of four codes (BITS / 2 bytes) into one float4, so that every store instruction of a wave
// covers 1 KiB of consecutive output; a workgroup works on contiguous chunks of UNROLL x kThreads groups
// with UNROLL loads in flight, whole chunks without bounds checks.
template <int BITS>
__device__ __forceinline__ uint32_t load_code_group(const uint8_t *__restrict__ codes, size_t g)
{
    if (BITS == 8) return __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(codes) + g);
    if (BITS == 4) return __builtin_nontemporal_load(reinterpret_cast<const uint16_t *>(codes) + g);
    if (BITS == 2) return __builtin_nontemporal_load(codes + g);
    const uint8_t *p = codes + g * 3;
    return p[0] | (p[1] << 8) | (p[2] << 16);
}

template <int BITS>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const uint8_t *__restrict__ codes, size_t n,
                                                              int is_signed, const float *__restrict__ scale,
                                                              float *__restrict__ y)
{
    __shared__ float lut[1 << BITS];
    const float s = *scale;
    for (int c = threadIdx.x; c < (1 << BITS); c += kThreads) lut[c] = s * code_value(c, BITS, is_signed);
    __syncthreads();
    constexpr int UNROLL = 4;
    constexpr uint32_t kMask = (1u << BITS) - 1;
    const size_t groups = n / 4;
    f32x4 *y4 = reinterpret_cast<f32x4 *>(y);
    auto expand = [&](uint32_t w) {
        return f32x4{lut[w & kMask], lut[(w >> BITS) & kMask], lut[(w >> (2 * BITS)) & kMask], lut[(w >> (3 * BITS)) & kMask]};
    };
    constexpr size_t per_block = (size_t)kThreads * UNROLL;
    for (size_t base = (size_t)blockIdx.x * per_block; base < groups; base += (size_t)gridDim.x * per_block) {
        const size_t i = base + threadIdx.x;
        uint32_t w[UNROLL];
        if (base + per_block <= groups) {                              // uniform: a whole chunk
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) w[u] = load_code_group<BITS>(codes, i + u * kThreads);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) __builtin_nontemporal_store(expand(w[u]), y4 + i + u * kThreads);
        } else {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) w[u] = (i + u * kThreads < groups) ? load_code_group<BITS>(codes, i + u * kThreads) : 0u;
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                if (i + u * kThreads < groups) __builtin_nontemporal_store(expand(w[u]), y4 + i + u * kThreads);
        }
    }
    // remainder (< 4 elements), one thread
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        for (size_t j = groups * 4; j < n; ++j) {
            const size_t bit = j * BITS;
            uint32_t w = codes[bit >> 3];
            if ((bit & 7) + BITS > 8) w |= (uint32_t)codes[(bit >> 3) + 1] << 8;
            y[j] = lut[(w >> (bit & 7)) & kMask];
        }
    }
}

static int grid_for(size_t work_items, int per_block, int max_blocks)
{
    size_t b = (work_items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > (size_t)max_blocks) b = max_blocks;
    return (int)b;
}

template <int BITS, bool SIGNED, int UNROLL>
static void launch_quantize_u(const float *x, size_t n, const float *scale, uint8_t *out, hipStream_t st,
                              float inv_vmax, float *scale_out)
{
    int *err = async_error_word();
    if (!err) { note_hip(hipErrorInvalidSymbol); return; }         // the entry point then reports DYBIT_ERR_HIP
    if (BITS == 6) {
        const size_t n16 = n / 16;
        if (n16) hipLaunchKernelGGL((quantize6_kernel<SIGNED, UNROLL>),
                                    dim3(grid_for(4 * n16, kThreads * UNROLL, 256 * DYBIT_QUANT_BLOCKS_PER_CU)), dim3(kThreads), 0, st,
                                    x, 4 * n16, scale, out, inv_vmax, scale_out, err);
        const size_t first = n16 * 16;
        if (first < n) {
            const size_t groups = (n - first + 3) / 4;
            hipLaunchKernelGGL((quantize_tail_kernel<BITS, SIGNED>), dim3((unsigned)groups), dim3(1), 0, st, x, first, n, scale, out,
                               inv_vmax, scale_out, err);
        }
    } else {
        const size_t n4 = n / 4;
        if (n4) hipLaunchKernelGGL((quantize_kernel<BITS == 6 ? 8 : BITS, SIGNED, UNROLL>),
                                   dim3(grid_for(n4, kThreads * UNROLL, 256 * DYBIT_QUANT_BLOCKS_PER_CU)), dim3(kThreads), 0, st, x, n4, scale, out, inv_vmax, scale_out, err);
        if (n4 * 4 < n)
            hipLaunchKernelGGL((quantize_tail_kernel<BITS, SIGNED>), dim3(1), dim3(1), 0, st, x, n4 * 4, n, scale, out, inv_vmax, scale_out, err);
    }
}

template <int BITS, bool SIGNED>
static void launch_quantize(const float *x, size_t n, const float *scale, uint8_t *out, hipStream_t st,
                            float inv_vmax = 0.0f, float *scale_out = nullptr)
{
    if (n / 4 < kQuantSmall) launch_quantize_u<BITS, SIGNED, DYBIT_QUANT_UNROLL_SMALL>(x, n, scale, out, st, inv_vmax, scale_out);
    else launch_quantize_u<BITS, SIGNED, DYBIT_QUANT_UNROLL>(x, n, scale, out, st, inv_vmax, scale_out);
}

}  // namespace dybit

using namespace dybit;

extern "C" dybit_status dybit_absmax_scale(const float *x, size_t n, dybit_fmt f, float *scale_out,
                                           dybit_stream stream)
{
    dybit_status st = check_fmt(f);
    if (st != DYBIT_OK) return st;
    if (!scale_out || (!x && n)) return DYBIT_ERR_NULL;
    if (!aligned16(x)) return DYBIT_ERR_ALIGNMENT;
    hipStream_t hs = (hipStream_t)stream;
    hipLaunchKernelGGL(absmax_init_kernel, dim3(1), dim3(1), 0, hs, scale_out);
    if (n) hipLaunchKernelGGL(absmax_kernel, dim3(grid_for(n / 4 + 1, kThreads * 4, 256 * 4)), dim3(kThreads), 0, hs, x, n, scale_out);
    const int m = mag_bits(f.bits, f.is_signed);
    hipLaunchKernelGGL(absmax_finish_kernel, dim3(1), dim3(1), 0, hs, scale_out, 1.0f / (float)(1u << (m - 1)));
    return launch_status();
}

extern "C" dybit_status dybit_scale_from_absmax(const float *absmax, dybit_fmt f, float *scale_out, dybit_stream stream)
{
    dybit_status st = check_fmt(f);
    if (st != DYBIT_OK) return st;
    if (!absmax || !scale_out) return DYBIT_ERR_NULL;
    const int m = mag_bits(f.bits, f.is_signed);
    hipLaunchKernelGGL(absmax_to_scale_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, absmax, scale_out,
                       1.0f / (float)(1u << (m - 1)));
    return launch_status();
}

extern "C" dybit_status dybit_quantize(const float *x, size_t n, dybit_fmt f, const float *scale,
                                       uint8_t *codes_out, dybit_stream stream)
{
    dybit_status st = check_fmt(f);
    if (st != DYBIT_OK) return st;
    if (!scale || ((!x || !codes_out) && n)) return DYBIT_ERR_NULL;
    if (!aligned16(x) || !aligned16(codes_out)) return DYBIT_ERR_ALIGNMENT;
    if (n == 0) return DYBIT_OK;
    hipStream_t hs = (hipStream_t)stream;
#define DYBIT_Q(B, S) launch_quantize<B, S>(x, n, scale, codes_out, hs)
    switch (f.bits * 2 + f.is_signed) {
        case 4: DYBIT_Q(2, false); break;   case 5: DYBIT_Q(2, true); break;
        case 8: DYBIT_Q(4, false); break;   case 9: DYBIT_Q(4, true); break;
        case 12: DYBIT_Q(6, false); break;  case 13: DYBIT_Q(6, true); break;
        case 16: DYBIT_Q(8, false); break;  case 17: DYBIT_Q(8, true); break;
    }
#undef DYBIT_Q
    return launch_status();
}

extern "C" dybit_status dybit_quantize_absmax(const float *x, size_t n, dybit_fmt f, const float *absmax, float *scale_out,
                                              uint8_t *codes_out, dybit_stream stream)
{
    dybit_status st = check_fmt(f);
    if (st != DYBIT_OK) return st;
    if (!absmax || !scale_out || ((!x || !codes_out) && n)) return DYBIT_ERR_NULL;
    if (absmax == scale_out) return DYBIT_ERR_INVALID_ARG;              // every block reads the maximum; one thread writes the scale
    if (!aligned16(x) || !aligned16(codes_out)) return DYBIT_ERR_ALIGNMENT;
    hipStream_t hs = (hipStream_t)stream;
    const float inv_vmax = 1.0f / (float)(1u << (mag_bits(f.bits, f.is_signed) - 1));
    if (n == 0) {                                                       // nothing to encode: the scale is still produced
        hipLaunchKernelGGL(absmax_to_scale_kernel, dim3(1), dim3(1), 0, hs, absmax, scale_out, inv_vmax);
        return launch_status();
    }
#define DYBIT_Q(B, S) launch_quantize<B, S>(x, n, absmax, codes_out, hs, inv_vmax, scale_out)
    switch (f.bits * 2 + f.is_signed) {
        case 4: DYBIT_Q(2, false); break;   case 5: DYBIT_Q(2, true); break;
        case 8: DYBIT_Q(4, false); break;   case 9: DYBIT_Q(4, true); break;
        case 12: DYBIT_Q(6, false); break;  case 13: DYBIT_Q(6, true); break;
        case 16: DYBIT_Q(8, false); break;  case 17: DYBIT_Q(8, true); break;
    }
#undef DYBIT_Q
    return launch_status();
}

extern "C" dybit_status dybit_quantize_rows(const float *x, int64_t rows, int64_t cols, dybit_fmt f, float *scales_out,
                                            uint8_t *codes_out, dybit_stream stream)
{
    dybit_status st = check_fmt(f);
    if (st != DYBIT_OK) return st;
    if (rows < 0 || cols < 0 || rows > 0x7fffffff) return DYBIT_ERR_INVALID_ARG;
    if ((cols * f.bits) % 8) return DYBIT_ERR_ALIGNMENT;
    if (rows == 0) return DYBIT_OK;
    if (!scales_out || ((!x || !codes_out) && cols)) return DYBIT_ERR_NULL;
    const float inv_vmax = 1.0f / (float)(1u << (mag_bits(f.bits, f.is_signed) - 1));
    int *err = async_error_word();
    if (!err) return DYBIT_ERR_HIP;
#define DYBIT_QR(B, S) hipLaunchKernelGGL((quantize_rows_kernel<B, S>), dim3((unsigned)rows), dim3(kThreads), 0, (hipStream_t)stream, \
                                          x, cols, inv_vmax, scales_out, codes_out, err)
    switch (f.bits * 2 + f.is_signed) {
        case 4: DYBIT_QR(2, false); break;   case 5: DYBIT_QR(2, true); break;
        case 8: DYBIT_QR(4, false); break;   case 9: DYBIT_QR(4, true); break;
        case 12: DYBIT_QR(6, false); break;  case 13: DYBIT_QR(6, true); break;
        case 16: DYBIT_QR(8, false); break;  case 17: DYBIT_QR(8, true); break;
    }
#undef DYBIT_QR
    return launch_status();
}

extern "C" dybit_status dybit_quantize_cols(const float *x, int64_t rows, int64_t cols, dybit_fmt f, float *scales_out,
                                            uint8_t *codes_out, dybit_stream stream)
{
    dybit_status st = check_fmt(f);
    if (st != DYBIT_OK) return st;
    if (rows < 0 || cols < 0 || rows > (1 << 30) || cols > (1 << 30)) return DYBIT_ERR_INVALID_ARG;
    if ((cols * f.bits) % 8) return DYBIT_ERR_ALIGNMENT;
    if (cols == 0) return DYBIT_OK;
    if (!scales_out || ((!x || !codes_out) && rows)) return DYBIT_ERR_NULL;
    hipStream_t hs = (hipStream_t)stream;
    const float inv_vmax = 1.0f / (float)(1u << (mag_bits(f.bits, f.is_signed) - 1));
    hipLaunchKernelGGL(col_scale_kernel, dim3((unsigned)((cols + 63) / 64)), dim3(kThreads), 0, hs, x, rows, cols, inv_vmax, scales_out);
    const int64_t groups = rows * cols / (f.bits == 8 ? 1 : f.bits == 4 ? 2 : 4);
    int *err = async_error_word();
    if (!err) return DYBIT_ERR_HIP;
    if (groups) {
        const dim3 grid((unsigned)((groups + kThreads - 1) / kThreads));
#define DYBIT_QC(B, S) hipLaunchKernelGGL((quantize_cols_kernel<B, S>), grid, dim3(kThreads), 0, hs, x, cols, groups, scales_out, codes_out, err)
        switch (f.bits * 2 + f.is_signed) {
            case 4: DYBIT_QC(2, false); break;   case 5: DYBIT_QC(2, true); break;
            case 8: DYBIT_QC(4, false); break;   case 9: DYBIT_QC(4, true); break;
            case 12: DYBIT_QC(6, false); break;  case 13: DYBIT_QC(6, true); break;
            case 16: DYBIT_QC(8, false); break;  case 17: DYBIT_QC(8, true); break;
        }
#undef DYBIT_QC
    }
    return launch_status();
}

extern "C" dybit_status dybit_quantize_pad(const float *x, int64_t rows, int64_t cols, int64_t cols_padded, dybit_fmt f,
                                           const float *scale, uint8_t *codes_out, dybit_stream stream)
{
    dybit_status st = check_fmt(f);
    if (st != DYBIT_OK) return st;
    if (rows < 0 || cols < 1 || cols_padded < cols || cols_padded > (1 << 24) || rows > ((int64_t)1 << 40)) return DYBIT_ERR_INVALID_ARG;
    if (cols_padded % 4) return DYBIT_ERR_ALIGNMENT;
    if (rows == 0) return DYBIT_OK;
    if (!x || !scale || !codes_out) return DYBIT_ERR_NULL;
    int *err = async_error_word();
    if (!err) return DYBIT_ERR_HIP;
    const int64_t groups = rows * (cols_padded / 4);
    const dim3 grid((unsigned)((groups + kThreads - 1) / kThreads < 256 * 64 ? (groups + kThreads - 1) / kThreads : 256 * 64));
#define DYBIT_QP(B, S) hipLaunchKernelGGL((quantize_pad_kernel<B, S>), grid, dim3(kThreads), 0, (hipStream_t)stream, \
                                          x, (int)cols, (int)(cols_padded / 4), groups, scale, codes_out, err)
    switch (f.bits * 2 + f.is_signed) {
        case 4: DYBIT_QP(2, false); break;   case 5: DYBIT_QP(2, true); break;
        case 8: DYBIT_QP(4, false); break;   case 9: DYBIT_QP(4, true); break;
        case 12: DYBIT_QP(6, false); break;  case 13: DYBIT_QP(6, true); break;
        case 16: DYBIT_QP(8, false); break;  case 17: DYBIT_QP(8, true); break;
    }
#undef DYBIT_QP
    return launch_status();
}

extern "C" dybit_status dybit_fake_quant_bwd(const float *x, const float *grad_out, size_t n, dybit_fmt f, const float *scale,
                                             float *grad_in, dybit_stream stream)
{
    dybit_status st = check_fmt(f);
    if (st != DYBIT_OK) return st;
    if (!scale || ((!x || !grad_out || !grad_in) && n)) return DYBIT_ERR_NULL;
    if (!aligned16(x) || !aligned16(grad_out) || !aligned16(grad_in)) return DYBIT_ERR_ALIGNMENT;
    if (n == 0) return DYBIT_OK;
    const float vmax = (float)(1u << (mag_bits(f.bits, f.is_signed) - 1));
    const int grid = grid_for(n / 4 + 1, kThreads * 2, 256 * 64);
    int *err = async_error_word();
    if (!err) return DYBIT_ERR_HIP;
    hipLaunchKernelGGL(fake_quant_bwd_kernel, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, x, grad_out, n, scale, vmax,
                       f.is_signed, grad_in, err);
    return launch_status();
}

extern "C" dybit_status dybit_fake_quant(const float *x, size_t n, dybit_fmt f, const float *scale, float *y_out,
                                         dybit_stream stream)
{
    dybit_status st = check_fmt(f);
    if (st != DYBIT_OK) return st;
    if (!scale || ((!x || !y_out) && n)) return DYBIT_ERR_NULL;
    if (!aligned16(x) || !aligned16(y_out)) return DYBIT_ERR_ALIGNMENT;
    if (n == 0) return DYBIT_OK;
    hipStream_t hs = (hipStream_t)stream;
    const int grid = grid_for(n / 4 + 1, kThreads * 4, 256 * DYBIT_QUANT_BLOCKS_PER_CU);
    int *err = async_error_word();
    if (!err) return DYBIT_ERR_HIP;
#define DYBIT_FQ(B, S) hipLaunchKernelGGL((fake_quant_kernel<B, S, 4>), dim3(grid), dim3(kThreads), 0, hs, x, n, scale, y_out, err)
    switch (f.bits * 2 + f.is_signed) {
        case 4: DYBIT_FQ(2, false); break;   case 5: DYBIT_FQ(2, true); break;
        case 8: DYBIT_FQ(4, false); break;   case 9: DYBIT_FQ(4, true); break;
        case 12: DYBIT_FQ(6, false); break;  case 13: DYBIT_FQ(6, true); break;
        case 16: DYBIT_FQ(8, false); break;  case 17: DYBIT_FQ(8, true); break;
    }
#undef DYBIT_FQ
    return launch_status();
}

extern "C" dybit_status dybit_dequantize(const uint8_t *codes, size_t n, dybit_fmt f, const float *scale,
                                         float *y_out, dybit_stream stream)
{
    dybit_status st = check_fmt(f);
    if (st != DYBIT_OK) return st;
    if (!scale || ((!codes || !y_out) && n)) return DYBIT_ERR_NULL;
    if (!aligned16(codes) || !aligned16(y_out)) return DYBIT_ERR_ALIGNMENT;
    if (n == 0) return DYBIT_OK;
    hipStream_t hs = (hipStream_t)stream;
    const int grid = grid_for(n / 4 + 1, kThreads * 4, 256 * 16);
    switch (f.bits) {
        case 2: hipLaunchKernelGGL((dequantize_kernel<2>), dim3(grid), dim3(kThreads), 0, hs, codes, n, f.is_signed, scale, y_out); break;
        case 4: hipLaunchKernelGGL((dequantize_kernel<4>), dim3(grid), dim3(kThreads), 0, hs, codes, n, f.is_signed, scale, y_out); break;
        case 6: hipLaunchKernelGGL((dequantize_kernel<6>), dim3(grid), dim3(kThreads), 0, hs, codes, n, f.is_signed, scale, y_out); break;
        case 8: hipLaunchKernelGGL((dequantize_kernel<8>), dim3(grid), dim3(kThreads), 0, hs, codes, n, f.is_signed, scale, y_out); break;
    }
    return launch_status();
}

namespace dybit {
namespace {
thread_local int *tl_error_word = nullptr;        // caller-owned word of this host thread, or NULL: the library's
}
// Device word that receives asynchronous errors of the calls this host thread makes: the caller's
// (dybit_set_async_error_word), else the library's own on the current device (each device has its copy;
// the address is looked up once per device).
int *async_error_word()
{
    if (tl_error_word) return tl_error_word;
    static int *cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    if (!cached[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_async_error)) != hipSuccess) return nullptr;
        cached[dev] = static_cast<int *>(ptr);
    }
    return cached[dev];
}
}  // namespace dybit

extern "C" dybit_status dybit_set_async_error_word(int32_t *device_word)
{
    if (reinterpret_cast<uintptr_t>(device_word) & 3u) return DYBIT_ERR_ALIGNMENT;
    dybit::tl_error_word = device_word;
    return DYBIT_OK;
}

extern "C" dybit_status dybit_get_last_async_error(int32_t *flag_out, dybit_stream stream)
{
    if (!flag_out) return DYBIT_ERR_NULL;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return DYBIT_ERR_HIP;
    int v = 0, zero = 0;
    if (hipMemcpyFromSymbol(&v, HIP_SYMBOL(g_async_error), sizeof(int)) != hipSuccess) return DYBIT_ERR_HIP;
    if (v && hipMemcpyToSymbol(HIP_SYMBOL(g_async_error), &zero, sizeof(int)) != hipSuccess) return DYBIT_ERR_HIP;
    *flag_out = v;
    return DYBIT_OK;
}
