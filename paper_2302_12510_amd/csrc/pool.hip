// Max pooling on packed DyBit codes (Sec. III-B: between layers the activations exist as codes only).
// The encoder is monotone -- a larger value never gets a code of smaller value -- so the code of the
// maximum of a window equals the maximum, by value, of the window's codes: pooling the codes gives bit for
// bit what quantizing the pooled fp32 tensor under the same scale would give, at 1/8 .. 1/4 of the bytes.
//
// Layout: NHWC, a pixel is C codes packed along C (C * bits a multiple of 32).  One thread owns one
// 32-bit word of one output pixel (32 / bits channels) and walks the k x k window, skipping the taps outside
// the image (a window always has one inside: 2 pad <= k).  The word is split into planes that hold two fields
// each in the halves of a register (plane p: fields p and p + 16 / bits), so that one packed 16-bit maximum
// serves two channels.  Unsigned codes order like their values.  Sign-magnitude codes are first mapped to
// offset keys (non-negative: code + 2^(bits-1); negative: 2^(bits-1) - 1 - magnitude), which order like the
// values, and mapped back at the end; value zero is always written as the all-zero code.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dybit.h"
#include "dybit_host.h"

namespace dybit {
namespace {

constexpr int kThreads = 256;

struct PoolArgs {
    const uint32_t *x;
    uint32_t *y;
    int H, W, Ho, Wo, k, stride, pad;
    int words;                    // 32-bit words per pixel
    int64_t total;                // output words
    int is_signed;
};

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

template <int BITS>
__global__ __launch_bounds__(kThreads) void maxpool_codes_kernel(const PoolArgs a)
{
    constexpr int PLANES = 16 / BITS;                               // fields per 16-bit half
    constexpr uint32_t kField = (1u << BITS) - 1u;
    constexpr uint32_t kPlane = kField | (kField << 16);            // field 0 of both halves
    constexpr uint32_t kSign = (1u << (BITS - 1)) * 0x00010001u, kMag = ((1u << (BITS - 1)) - 1u) * 0x00010001u;
    const bool is_signed = a.is_signed != 0;                        // uniform
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < a.total; i += (int64_t)gridDim.x * kThreads) {
        const int64_t pix = i / a.words;
        const int word = (int)(i - pix * a.words);
        const int wo = (int)(pix % a.Wo);
        const int64_t t = pix / a.Wo;
        const int ho = (int)(t % a.Ho);
        const int64_t b = t / a.Ho;
        const int h_lo = ho * a.stride - a.pad, w_lo = wo * a.stride - a.pad;
        uint32_t best[PLANES];
#pragma unroll
        for (int p = 0; p < PLANES; ++p) best[p] = 0u;              // the smallest key
        for (int r = max(h_lo, 0); r < min(h_lo + a.k, a.H); ++r) {
            const uint32_t *row = a.x + ((b * a.H + r) * a.W) * a.words + word;
            for (int s = max(w_lo, 0); s < min(w_lo + a.k, a.W); ++s) {
                const uint32_t w = row[(int64_t)s * a.words];
#pragma unroll
                for (int p = 0; p < PLANES; ++p) {
                    uint32_t c = (w >> (p * BITS)) & kPlane;
                    if (is_signed) {
                        const uint32_t sg = c & kSign;               // key = c ^ sign bit, magnitude inverted where the sign is set
                        c ^= kSign ^ (sg - (sg >> (BITS - 1)));
                    }
                    const u16x2 m = __builtin_elementwise_max(__builtin_bit_cast(u16x2, best[p]), __builtin_bit_cast(u16x2, c));
                    best[p] = __builtin_bit_cast(uint32_t, m);
                }
            }
        }
        uint32_t out = 0;
#pragma unroll
        for (int p = 0; p < PLANES; ++p) {
            uint32_t c = best[p];
            if (is_signed) {
                // keys >= 2^(bits-1) are the non-negative codes; below: negative, magnitude 2^(bits-1) - 1 - key,
                // and magnitude 0 (the negative zero) becomes the all-zero code
                const uint32_t pos = c & kSign;                      // set: non-negative
                const uint32_t neg = (pos ^ kSign) - ((pos ^ kSign) >> (BITS - 1));   // kMag where negative
                const uint32_t mag = (c ^ neg) & kMag;
                const uint32_t nz = (mag | (mag >> 1) | (mag >> 2) | (mag >> 3) | (mag >> 4) | (mag >> 5) | (mag >> 6)) & 0x00010001u;
                c = mag | ((pos ^ kSign) & (nz << (BITS - 1)));      // sign only with a non-zero magnitude
            }
            out |= c << (p * BITS);
        }
        a.y[i] = out;
    }
}

}  // namespace
}  // namespace dybit

using namespace dybit;

extern "C" dybit_status dybit_maxpool2d_codes(int64_t B, int64_t H, int64_t W, int64_t C,
                                              int32_t k, int32_t stride, int32_t pad,
                                              const uint8_t *X_codes, dybit_fmt fmt, uint8_t *Y_codes, dybit_stream stream)
{
    if (fmt.bits != 2 && fmt.bits != 4 && fmt.bits != 8) return DYBIT_ERR_UNSUPPORTED_BITS;
    if (fmt.is_signed != 0 && fmt.is_signed != 1) return DYBIT_ERR_INVALID_ARG;
    if (B < 0 || H < 1 || W < 1 || C < 1 || k < 1 || stride < 1 || pad < 0 || 2 * pad > k) return DYBIT_ERR_INVALID_ARG;
    if (H > (1 << 24) || W > (1 << 24) || H + 2 * (int64_t)pad < k || W + 2 * (int64_t)pad < k) return DYBIT_ERR_INVALID_ARG;
    if ((C * fmt.bits) % 32) return DYBIT_ERR_ALIGNMENT;
    if (B == 0) return DYBIT_OK;
    if (!X_codes || !Y_codes) return DYBIT_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(X_codes) | reinterpret_cast<uintptr_t>(Y_codes)) & 3u) return DYBIT_ERR_ALIGNMENT;
    PoolArgs a;
    a.x = reinterpret_cast<const uint32_t *>(X_codes);
    a.y = reinterpret_cast<uint32_t *>(Y_codes);
    a.H = (int)H; a.W = (int)W; a.k = k; a.stride = stride; a.pad = pad;
    a.Ho = (int)((H + 2 * pad - k) / stride + 1);
    a.Wo = (int)((W + 2 * pad - k) / stride + 1);
    a.words = (int)(C * fmt.bits / 32);
    a.total = B * a.Ho * a.Wo * a.words;
    a.is_signed = fmt.is_signed;
    const int64_t blocks = (a.total + kThreads - 1) / kThreads;
    const dim3 grid((unsigned)(blocks < 256 * 32 ? blocks : 256 * 32)), block(kThreads);
    hipStream_t st = (hipStream_t)stream;
    switch (fmt.bits) {
        case 2: hipLaunchKernelGGL(maxpool_codes_kernel<2>, grid, block, 0, st, a); break;
        case 4: hipLaunchKernelGGL(maxpool_codes_kernel<4>, grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL(maxpool_codes_kernel<8>, grid, block, 0, st, a); break;
    }
    return launch_status();
}
