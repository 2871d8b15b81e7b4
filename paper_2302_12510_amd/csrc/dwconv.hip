// Depthwise convolution on DyBit codes for gfx950 (the layer type of the depthwise-separable
// network of Sec. IV): Y[b,ho,wo,c] = sA sW sum_{r,s} x[b,hi,wi,c] w[r,s,c] (+ bias[c]) (ReLU).
//
// Nine multiply-adds per output and no contraction over channels: this is not matrix-core work.
// It is bound by the fp32 output (4 bytes per result against <= 1 byte of codes read), so the
// kernel is organised to keep the vector-ALU work per output low enough for the HBM rate:
// a workgroup owns an 8 x 8 (3 x 3 filter at stride 1: 8 x 16) patch of output pixels and 32 channels; it decodes the input patch
// (with its halo) and the filter taps of those channels ONCE into LDS as floats, then every thread
// accumulates four neighbouring channels of a pixel with 128-bit LDS reads -- each input code is
// decoded once per patch (a look-up in a small LDS table of the format's values) instead of once
// per tap.  The 3 x 3 filters at stride 1 and 2 have kernels of their own with the taps unrolled
// and held in registers; every other geometry runs the same code with run-time loops.  Image, filter and output are channel-innermost,
// so global loads (whole 32-bit words of codes) and stores (float4) are contiguous per pixel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "dybit_device.h"
#include "dybit_host.h"
#include "gemm_args.h"
#include "requant.h"

namespace dybit {
namespace {

constexpr int kThreads = 256;
constexpr int TH = 8, CG = 32;                     // rows of the output patch and channel group of a workgroup
// columns of the output patch: 16 for the 3 x 3 filter at stride 1 (the halo and the fixed work of a
// workgroup are shared by more outputs), 8 otherwise (a wider input patch would not leave room for
// several workgroups per compute unit)
constexpr int patch_width(int kh, int kw, int stride) { return (kh == 3 && kw == 3 && stride == 1) ? 16 : 8; }
constexpr int kMaxLdsBytes = 64 * 1024;
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct DwArgs {
    const uint32_t *X, *Wt;                        // packed codes, read as whole words
    const float *x_scale, *w_scale, *bias;
    float *Y;                                      // may be NULL when q_out is given
    uint32_t *absmax_bits;
    int w_per_channel;                             // w_scale holds one value per channel
    uint8_t *q_out;                                // optional write-back as DyBit codes, packed along C like the image
    const float *q_scale;
    int q_bits, q_signed;
    int *async_error;
    int B, H, W, C, Ho, Wo, kh, kw, stride, pad, relu;
    int a_bits, a_signed, w_bits, w_signed;
    int in_h, in_w;                                // extent of the input patch, halo included
    int tiles_h, tiles_w, groups;
};

// K: filter size when it is square and known at compile time (3), else 0; S: stride (1, 2) or 0.
// BA, BW: code widths of image and filter (2, 4 or 8).
template <int BA, int BW, int K, int S>
__global__ __launch_bounds__(kThreads) void dwconv_kernel(const DwArgs a)
{
    constexpr int TW = patch_width(K, K, S);
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int kh = K ? K : a.kh, kw = K ? K : a.kw, stride = S ? S : a.stride;
    const int in_h = (TH - 1) * stride + kh, in_w = (TW - 1) * stride + kw;
    float *tile = lds;                                           // [in_h * in_w][CG]
    float *taps = tile + (size_t)in_h * in_w * CG;               // [kh * kw][CG]
    float *lut_a = taps + (size_t)kh * kw * CG;                  // value of every code of the two formats
    float *lut_w = lut_a + (1 << BA);
    const int tid = threadIdx.x;
    int id = blockIdx.x;
    const int cg = id % a.groups; id /= a.groups;
    const int tw = id % a.tiles_w; id /= a.tiles_w;
    const int th = id % a.tiles_h;
    const int b = id / a.tiles_h;
    const int ho0 = th * TH, wo0 = tw * TW, c_first = cg * CG;

    if (tid < (1 << BA)) lut_a[tid] = code_value(tid, BA, a.a_signed);
    if (tid < (1 << BW)) lut_w[tid] = code_value(tid, BW, a.w_signed);
    __syncthreads();

    // Writes the values of the CPW codes of one word to consecutive floats, four at a time.
    auto expand = [&](uint32_t word, const float *lut, auto bits_tag, float *dst) {
        constexpr int BITS = decltype(bits_tag)::value, CPW = 32 / BITS;
#pragma unroll
        for (int j = 0; j < CPW; j += 4) {
            f32x4 v;
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = lut[(word >> ((j + u) * BITS)) & ((1u << BITS) - 1u)];
            *reinterpret_cast<f32x4 *>(dst + j) = v;
        }
    };
    // ---- stage the input patch: one item = one word of codes of one pixel (offsets inside one image fit 32 bits)
    {
        constexpr int WPP = CG * BA / 32, CPW = 32 / BA;                  // words per pixel and group, codes per word
        const int row_words = a.C * BA / 32;                              // words per pixel in the image
        const uint32_t *image = a.X + (int64_t)b * a.H * a.W * row_words + c_first * BA / 32;
        const int items = in_h * in_w * WPP;
        const int hi0 = ho0 * stride - a.pad, wi0 = wo0 * stride - a.pad;
        for (int it = tid; it < items; it += kThreads) {
            const int pix = it / WPP, wd = it % WPP;
            const int iy = pix / in_w, ix = pix - iy * in_w;
            const int hi = hi0 + iy, wi = wi0 + ix;
            const bool in = (unsigned)hi < (unsigned)a.H && (unsigned)wi < (unsigned)a.W && c_first + wd * CPW < a.C;
            const uint32_t word = in ? image[(hi * a.W + wi) * row_words + wd] : 0u;
            expand(word, lut_a, std::integral_constant<int, BA>{}, tile + pix * CG + wd * CPW);   // code 0 is 0.0: padding, channels past C
        }
    }
    // ---- stage the filter taps of the group's channels
    {
        constexpr int WPP = CG * BW / 32, CPW = 32 / BW;
        const int row_words = a.C * BW / 32;
        const int items = kh * kw * WPP;
        for (int it = tid; it < items; it += kThreads) {
            const int tap = it / WPP, wd = it % WPP;
            const bool in = c_first + wd * CPW < a.C;
            const uint32_t word = in ? a.Wt[tap * row_words + c_first * BW / 32 + wd] : 0u;
            expand(word, lut_w, std::integral_constant<int, BW>{}, taps + tap * CG + wd * CPW);
        }
    }
    __syncthreads();

    // ---- accumulate.  A thread's four channels are the same for all its outputs: their scales are read once.
    const int c_thread = c_first + (tid & (CG / 4 - 1)) * 4;
    f32x4 alpha;
    {
        const float sx = *a.x_scale;
        const bool pc = a.w_per_channel && c_thread < a.C;
#pragma unroll
        for (int u = 0; u < 4; ++u) alpha[u] = sx * (pc ? a.w_scale[c_thread + u] : a.w_scale[0]);
    }
    // optional write-back (Sec. III-B): the four results of a thread are four neighbouring codes of the
    // packed output pixel, i.e. 16 bits (4-bit formats) or one word (8-bit formats)
    Requant rq{};
    const bool wb = a.q_out != nullptr;
    if (wb) {
        rq = make_requant(a.q_scale, a.q_bits, a.q_signed);
        if (!rq.ok && blockIdx.x == 0 && tid == 0) *a.async_error = DYBIT_ERR_BAD_SCALE;   // no codes, flag the call
    }
    float mx = 0.0f;
    auto finish = [&](const f32x4 acc, const f32x4 bv, int64_t elem) {          // elem: index of the thread's first output value
        f32x4 y;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            y[u] = acc[u] * alpha[u] + bv[u];
            if (a.relu) y[u] = fmaxf(y[u], 0.0f);
            mx = fmaxf(mx, fabsf(y[u]));
        }
        if (a.Y) __builtin_nontemporal_store(y, reinterpret_cast<f32x4 *>(a.Y + elem));
        if (wb && rq.ok) {
            uint32_t w = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) w |= requant_code(y[u], rq) << (u * a.q_bits);
            if (a.q_bits == 8) *reinterpret_cast<uint32_t *>(a.q_out + elem) = w;
            else *reinterpret_cast<uint16_t *>(a.q_out + (elem >> 1)) = (uint16_t)w;
        }
    };
    if constexpr (K != 0) {
        // 3 x 3: a thread owns four neighbouring channels of one output column and R consecutive output
        // rows; the taps stay in registers and the window of input rows slides down, so that an input
        // row is read from LDS once per thread, not once per output row.
        constexpr int COLS = TW * (CG / 4), R = TH / (kThreads / COLS);
        const int col = tid % COLS, quad = col & (CG / 4 - 1), px = col / (CG / 4), py0 = (tid / COLS) * R;
        const int c = c_first + quad * 4, wo = wo0 + px;
        f32x4 wreg[K * K], win[K][K];
#pragma unroll
        for (int t = 0; t < K * K; ++t) wreg[t] = *reinterpret_cast<const f32x4 *>(taps + t * CG + quad * 4);
        const bool col_ok = wo < a.Wo && c < a.C;                 // C is a multiple of 4: a quad is inside or outside
        f32x4 bv = {0.f, 0.f, 0.f, 0.f};
        if (a.bias && col_ok) bv = *reinterpret_cast<const f32x4 *>(a.bias + c);
        int64_t elem = (((int64_t)b * a.Ho + ho0 + py0) * a.Wo + wo) * a.C + c;
        const float *origin = tile + ((py0 * S) * in_w + px * S) * CG + quad * 4;
#pragma unroll
        for (int i = 0; i < R; ++i) {
#pragma unroll
            for (int r = 0; r < K; ++r) {
                if (i > 0 && r + S < K) {                         // this input row was the previous output's row r + S
#pragma unroll
                    for (int q = 0; q < K; ++q) win[r][q] = win[r + S][q];
                } else {
#pragma unroll
                    for (int q = 0; q < K; ++q)
                        win[r][q] = *reinterpret_cast<const f32x4 *>(origin + ((i * S + r) * in_w + q) * CG);
                }
            }
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < K; ++r)
#pragma unroll
                for (int q = 0; q < K; ++q)
#pragma unroll
                    for (int u = 0; u < 4; ++u) acc[u] = fmaf(win[r][q][u], wreg[r * K + q][u], acc[u]);
            if (col_ok && ho0 + py0 + i < a.Ho) finish(acc, bv, elem);
            elem += (int64_t)a.Wo * a.C;
        }
    } else {
        // any other geometry: one item = four neighbouring channels of one output pixel, run-time loops
        const int quad = tid & (CG / 4 - 1);
        for (int it = tid; it < TH * TW * (CG / 4); it += kThreads) {
            const int pix = it / (CG / 4);
            const int py = pix / TW, px = pix % TW;
            const int ho = ho0 + py, wo = wo0 + px, c = c_first + quad * 4;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            const float *origin = tile + ((py * stride) * in_w + px * stride) * CG + quad * 4;
            for (int r = 0; r < kh; ++r)
                for (int q = 0; q < kw; ++q) {
                    const f32x4 x = *reinterpret_cast<const f32x4 *>(origin + (r * in_w + q) * CG);
                    const f32x4 w = *reinterpret_cast<const f32x4 *>(taps + (r * kw + q) * CG + quad * 4);
#pragma unroll
                    for (int u = 0; u < 4; ++u) acc[u] = fmaf(x[u], w[u], acc[u]);
                }
            if (ho < a.Ho && wo < a.Wo && c < a.C) {
                f32x4 bv = {0.f, 0.f, 0.f, 0.f};
                if (a.bias) bv = *reinterpret_cast<const f32x4 *>(a.bias + c);
                finish(acc, bv, (((int64_t)b * a.Ho + ho) * a.Wo + wo) * a.C + c);
            }
        }
    }
    if (a.absmax_bits) fold_absmax(a.absmax_bits, mx);           // every lane of every wave arrives here
}

template <int BA, int BW>
void launch_dw(const DwArgs &a, size_t lds_bytes, hipStream_t st, unsigned blocks)
{
    auto go = [&](auto kernel) {
        note_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kThreads), lds_bytes, st, a);
    };
    if (a.kh == 3 && a.kw == 3 && a.stride == 1) go(dwconv_kernel<BA, BW, 3, 1>);
    else if (a.kh == 3 && a.kw == 3 && a.stride == 2) go(dwconv_kernel<BA, BW, 3, 2>);
    else go(dwconv_kernel<BA, BW, 0, 0>);
}

}  // namespace
}  // namespace dybit

using namespace dybit;

static dybit_status dwconv_impl(int64_t B, int64_t H, int64_t W, int64_t C,
                                int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                                const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale, int32_t w_per_channel,
                                const float *bias, int32_t relu, float *Y, float *y_absmax,
                                dybit_fmt y_fmt, const float *y_scale, uint8_t *Y_codes, dybit_stream stream)
{
    dybit_status st = check_fmt(x_fmt);
    if (st == DYBIT_OK) st = check_fmt(w_fmt);
    if (st != DYBIT_OK) return st;
    if (x_fmt.bits == 6 || w_fmt.bits == 6) return DYBIT_ERR_UNSUPPORTED_BITS;      // whole codes per 32-bit word only
    if (B < 0 || H < 1 || W < 1 || C < 0 || kh < 1 || kw < 1 || stride < 1 || pad < 0 || (relu != 0 && relu != 1) ||
        H > (1 << 24) || W > (1 << 24) || C > (1 << 24) || kh > 64 || kw > 64 || stride > 64)
        return DYBIT_ERR_INVALID_ARG;
    if (H + 2 * (int64_t)pad < kh || W + 2 * (int64_t)pad < kw) return DYBIT_ERR_INVALID_ARG;
    if ((C * x_fmt.bits) % 32 || (C * w_fmt.bits) % 32) return DYBIT_ERR_ALIGNMENT;   // a pixel's codes are whole words
    if (w_per_channel != 0 && w_per_channel != 1) return DYBIT_ERR_INVALID_ARG;
    if (Y_codes) {
        if ((st = check_fmt(y_fmt)) != DYBIT_OK) return st;
        if (y_fmt.bits != 4 && y_fmt.bits != 8) return DYBIT_ERR_UNSUPPORTED_BITS;     // four codes of a thread are 16 or 32 bits
        if ((C * y_fmt.bits) % 32) return DYBIT_ERR_ALIGNMENT;
        if (!y_scale) return DYBIT_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(Y_codes) & 3u) return DYBIT_ERR_ALIGNMENT;
    }
    const int64_t Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
    const int TW = patch_width(kh, kw, stride);
    const int in_h = (TH - 1) * stride + kh, in_w = (TW - 1) * stride + kw;
    const int64_t lds_bytes = ((int64_t)in_h * in_w + (int64_t)kh * kw) * CG * 4 + 4 * ((1 << x_fmt.bits) + (1 << w_fmt.bits));
    if (lds_bytes > kMaxLdsBytes) return DYBIT_ERR_INVALID_ARG;                    // filter / stride too large for one patch
    if (H * W * (C * x_fmt.bits / 32) > 0x7fffffff || (int64_t)kh * kw * (C * w_fmt.bits / 32) > 0x7fffffff)
        return DYBIT_ERR_INVALID_ARG;                                              // offsets inside one image are 32-bit
    if (B == 0 || C == 0) return DYBIT_OK;
    if (!x_scale || !w_scale || !X_codes || !Wt_codes || (!Y && !Y_codes)) return DYBIT_ERR_NULL;
    if (!aligned16(X_codes) || !aligned16(Wt_codes) || !aligned16(Y) || (bias && !aligned16(bias))) return DYBIT_ERR_ALIGNMENT;
    clear_call_record();
    DwArgs a{};
    a.X = reinterpret_cast<const uint32_t *>(X_codes); a.Wt = reinterpret_cast<const uint32_t *>(Wt_codes);
    a.x_scale = x_scale; a.w_scale = w_scale; a.bias = bias; a.Y = Y;
    a.absmax_bits = reinterpret_cast<uint32_t *>(y_absmax);
    a.w_per_channel = w_per_channel;
    if (Y_codes) {
        a.q_out = Y_codes; a.q_scale = y_scale; a.q_bits = y_fmt.bits; a.q_signed = y_fmt.is_signed;
        a.async_error = async_error_word();
        if (!a.async_error) return DYBIT_ERR_HIP;
    }
    a.B = (int)B; a.H = (int)H; a.W = (int)W; a.C = (int)C; a.Ho = (int)Ho; a.Wo = (int)Wo;
    a.kh = kh; a.kw = kw; a.stride = stride; a.pad = pad; a.relu = relu;
    a.a_bits = x_fmt.bits; a.a_signed = x_fmt.is_signed; a.w_bits = w_fmt.bits; a.w_signed = w_fmt.is_signed;
    a.in_h = in_h; a.in_w = in_w;
    a.tiles_h = (int)((Ho + TH - 1) / TH); a.tiles_w = (int)((Wo + TW - 1) / TW); a.groups = (int)((C + CG - 1) / CG);
    const int64_t blocks = B * a.tiles_h * a.tiles_w * a.groups;
    if (blocks > 0x7fffffff || B > 0x7fffffff) return DYBIT_ERR_INVALID_ARG;
    hipStream_t hs = (hipStream_t)stream;
#define DYBIT_DW(BA, BW) launch_dw<BA, BW>(a, (size_t)lds_bytes, hs, (unsigned)blocks)
    switch (x_fmt.bits * 16 + w_fmt.bits) {
        case 0x22: DYBIT_DW(2, 2); break;  case 0x24: DYBIT_DW(2, 4); break;  case 0x28: DYBIT_DW(2, 8); break;
        case 0x42: DYBIT_DW(4, 2); break;  case 0x44: DYBIT_DW(4, 4); break;  case 0x48: DYBIT_DW(4, 8); break;
        case 0x82: DYBIT_DW(8, 2); break;  case 0x84: DYBIT_DW(8, 4); break;  case 0x88: DYBIT_DW(8, 8); break;
    }
#undef DYBIT_DW
    return launch_status();
}

extern "C" dybit_status dybit_dwconv2d(int64_t B, int64_t H, int64_t W, int64_t C,
                                       int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                       const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                                       const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale,
                                       const float *bias, int32_t relu, float *Y, float *y_absmax, dybit_stream stream)
{
    if (!Y && B && C) return DYBIT_ERR_NULL;
    return dwconv_impl(B, H, W, C, kh, kw, stride, pad, X_codes, x_fmt, x_scale, Wt_codes, w_fmt, w_scale, 0, bias, relu,
                       Y, y_absmax, dybit_fmt{0, 0}, nullptr, nullptr, stream);
}

extern "C" dybit_status dybit_dwconv2d_wb(int64_t B, int64_t H, int64_t W, int64_t C,
                                          int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                          const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                                          const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale, int32_t w_per_channel,
                                          const float *bias, int32_t relu, float *Y, float *y_absmax,
                                          dybit_fmt y_fmt, const float *y_scale, uint8_t *Y_codes, dybit_stream stream)
{
    return dwconv_impl(B, H, W, C, kh, kw, stride, pad, X_codes, x_fmt, x_scale, Wt_codes, w_fmt, w_scale, w_per_channel, bias, relu,
                       Y, y_absmax, y_fmt, y_scale, Y_codes, stream);
}
