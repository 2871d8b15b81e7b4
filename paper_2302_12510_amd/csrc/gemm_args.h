// Argument block shared by the DyBit matrix-product kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dybit {

struct GemmArgs {
    int64_t M, N, K;                 // conv: M = B*Ho*Wo, N = Cout, K = kh*kw*Cin
    const uint8_t *A, *W;            // packed codes, K-contiguous rows (conv: NHWC image / [Cout][kh][kw][Cin])
    int a_signed, w_signed;
    const float *a_scale, *w_scale, *bias;
    int relu;
    float *C;
    int64_t ldc;
    // convolution geometry (conv only)
    int H, Wd, Cin, Ho, Wo, kh, kw, stride, pad;
    int64_t a_bytes, w_bytes;        // sizes of the two code buffers
};

// Tiled MFMA kernels for 4- and 8-bit operands with signed weights: the large-tile kernel
// (gemm_fast.hip, 256 x 256) and the mid-size-tile kernel (gemm_mid.hip, 128 x 128), one
// translation unit per weight format.  a_bits is 4 or 8; signedness comes from g.
bool launch_gemm_fast_w0(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);   // W 4-bit signed
bool launch_gemm_fast_w2(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);   // W 8-bit signed
bool launch_gemm_mid_w0(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_mid_w2(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);

// Picks a tiled kernel for the problem (gemm_dispatch.cpp).  Returns false when the problem does
// not meet their preconditions; the caller then uses the general kernel.
bool launch_gemm_tiled(const GemmArgs &g, int a_bits, int w_bits, bool conv, hipStream_t st);

}  // namespace dybit
