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

// Large-tile kernel for 4- and 8-bit operands (gemm_fast.hip).  Returns false when the
// problem does not meet its preconditions; the caller then uses the general kernel.
bool launch_gemm_fast(const GemmArgs &g, int a_bits, int w_bits, bool conv, hipStream_t st);

}  // namespace dybit
