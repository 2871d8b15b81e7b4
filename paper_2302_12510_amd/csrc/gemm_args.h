// Argument block shared by the DyBit matrix-product kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#ifndef DYBIT_WB
#define DYBIT_WB 0
#endif
#if DYBIT_WB
#define DYBIT_WB_NAME(name) name##_wb
#else
#define DYBIT_WB_NAME(name) name
#endif

namespace dybit {

constexpr bool kWriteBack = DYBIT_WB != 0;

struct GemmArgs {
    int64_t M, N, K;                 // conv: M = B*Ho*Wo, N = Cout, K = kh*kw*Cin
    const uint8_t *A, *W;            // packed codes, K-contiguous rows (conv: NHWC image / [Cout][kh][kw][Cin])
    int a_signed, w_signed;
    const float *a_scale, *w_scale, *bias;
    int w_per_channel;               // 0: *w_scale is the scale of the whole tensor; 1: w_scale[n] per output column n
    const float *residual;           // optional: fp32 tensor laid out like C (same ldc), added before the ReLU
    // the shortcut as DyBit codes instead (write-back build only; at most one of the two forms): M rows of
    // res_row_bytes bytes holding N codes of res_bits bits (4, 6 or 8), value = *res_scale * value(code)
    const uint8_t *res_codes;
    const float *res_scale;
    int res_bits, res_signed;
    int64_t res_row_bytes;
    int relu;
    uint32_t *absmax_bits;           // optional: running max |C| of the written values, as float bits (atomic max)
    float *C;                        // may be NULL when q_out is given
    int64_t ldc;
    // optional write-back of the result as DyBit codes: M rows of q_row_bytes bytes (N codes, whole 32-bit words)
    uint8_t *q_out;
    const float *q_scale;
    int q_bits, q_signed;
    int64_t q_row_bytes;
    int *async_error;                // device word that receives DYBIT_ERR_BAD_SCALE when *q_scale is unusable
    // convolution geometry (conv only)
    int H, Wd, Cin, Ho, Wo, kh, kw, stride, pad;
    int pix_bytes;                   // bytes from a pixel to the next one in the image: Cin * bits / 8, or more when A
                                     // points at one channel group of a wider image (grouped convolution)
    int64_t a_bytes, w_bytes;        // sizes of the two code buffers
};

// Overrides of the automatic kernel choice (0 = automatic everywhere).  They start from the
// environment, read once when the library is first used (DYBIT_GEMM_KERNEL, DYBIT_GEMM_MFMA,
// DYBIT_MID_TILE, DYBIT_MID_KGROUPS, DYBIT_GEMM_WS), and change only through dybit_set_option.
struct DispatchOptions {
    int kernel;        // 0 automatic, else DYBIT_FORCE_*
    int mfma_f16;      // 1: pairs of 4- and 2-bit operands stay on the fp16 kernels
    int mid_tile;      // 0 automatic, 64 or 128: tile of the fp8-path kernel when it is not the 256 x 256 one
    int mid_kgroups;   // 0 automatic, 1 or 2: k-groups of the 128 x 128 kernels
    int ws_off;        // 1: the weight-stationary kernel is left out of the automatic choice
};
enum { DYBIT_FORCE_GENERAL = 1, DYBIT_FORCE_MID = 2, DYBIT_FORCE_LARGE = 3, DYBIT_FORCE_WS = 4 };
DispatchOptions dispatch_options();
// Record of the kernel a launch function started, per host thread (dybit_last_gemm_kernel reads it),
// and of a HIP error met on the way (hipFuncSetAttribute, ...), which the entry point then reports.
void note_kernel(int id);
void note_hip(hipError_t e);
void clear_call_record();          // an entry point calls this first
hipError_t take_hip_error();       // ... and this last: the first error noted since, or hipSuccess

// Tiled MFMA kernels for 4- and 8-bit operands with signed weights: the large-tile kernel
// (gemm_fast.hip, 256 x 256) and the mid-size-tile kernel (gemm_mid.hip, 128 x 128), one
// translation unit per weight format.  a_bits is 4 or 8; signedness comes from g.
// Every kernel source is compiled twice: plain, and with DYBIT_WB=1 as the write-back build whose
// epilogue also encodes the results (g.q_out must then be set); those entry points end in _wb.
bool launch_gemm_fast_w0(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);   // W 4-bit signed
bool launch_gemm_fast_w2(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);   // W 8-bit signed
bool launch_gemm_fast_w4(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);   // W 6-bit signed
bool launch_gemm_fast_w6(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);   // W 2-bit signed; a_bits 2, 4, 6 or 8 for all four; false:
                                                                                      // K (Cin) is not a multiple of 128 while an operand is 2- or 6-bit
bool launch_gemm_mid_w0(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_mid_w2(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_mid_w4(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);    // W 6-bit signed
bool launch_gemm_mid_w6(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);    // W 2-bit signed; a_bits 2, 4, 6 or 8 for all four
bool launch_gemm_fast_w0_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_fast_w2_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_fast_w4_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_fast_w6_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_mid_w0_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_mid_w2_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_mid_w4_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_mid_w6_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);

// Weight-stationary kernel (gemm_ws.hip) for layers whose decoded weight matrix fits the LDS of a
// compute unit (N <= 128, N rounded up to 64 or 128 rows of 2 K + 16 bytes within 160 KiB); one
// translation unit per weight format as above.  Returns false when the weights do not fit.
bool launch_gemm_ws_w0(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_ws_w2(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_ws_w4(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_ws_w6(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_ws_w0_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_ws_w2_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_ws_w4_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);
bool launch_gemm_ws_w6_wb(const GemmArgs &g, int a_bits, bool conv, hipStream_t st);

// fp8 matrix path for pairs of 4-bit formats with signed weights (gemm_f8.hip): the 256 x 256 tile
// when `large`, else the 128 x 128 tile.
bool launch_gemm_f8_w0(const GemmArgs &g, int a_bits, bool conv, bool large, hipStream_t st);      // W 4-bit signed
bool launch_gemm_f8_w6(const GemmArgs &g, int a_bits, bool conv, bool large, hipStream_t st);      // W 2-bit signed
bool launch_gemm_f8_w0_wb(const GemmArgs &g, int a_bits, bool conv, bool large, hipStream_t st);
bool launch_gemm_f8_w6_wb(const GemmArgs &g, int a_bits, bool conv, bool large, hipStream_t st);

// General kernel (gemm.hip): any format pair and shape.  mode: 0 operands fetched code by code;
// 1 operands are 16-byte aligned and K (convolution: Cin) is a multiple of 16; 2 (convolution
// only) aligned operands, Cin divides 16 and kw * Cin is a multiple of 16, tensor below 2 GiB.
void launch_gemm_general(const GemmArgs &g, int a_bits, int w_bits, bool conv, int mode, hipStream_t st);
void launch_gemm_general_wb(const GemmArgs &g, int a_bits, int w_bits, bool conv, int mode, hipStream_t st);
// the write-back build's kernels, one translation unit per activation width (gemm_dispatch.cpp joins them)
void launch_gemm_general_a2_wb(const GemmArgs &g, int w_bits, bool conv, int mode, hipStream_t st);
void launch_gemm_general_a4_wb(const GemmArgs &g, int w_bits, bool conv, int mode, hipStream_t st);
void launch_gemm_general_a6_wb(const GemmArgs &g, int w_bits, bool conv, int mode, hipStream_t st);
void launch_gemm_general_a8_wb(const GemmArgs &g, int w_bits, bool conv, int mode, hipStream_t st);

// Picks a tiled kernel for the problem (gemm_dispatch.cpp).  Returns false when the problem does
// not meet their preconditions; the caller then uses the general kernel.
bool launch_gemm_tiled(const GemmArgs &g, int a_bits, int w_bits, bool conv, hipStream_t st);

// Folds a lane's maximum of |c| into the running maximum: wave reduction, then at most one atomic
// per wave.  Non-negative floats order like their bit patterns; fmaxf has already dropped NaNs.
// Atomics on one address serialise (about 10 ns each), and a large layer has tens of thousands of
// waves, so a wave first reads the word (at device scope, from L2) and only competes when it would
// raise it: the running maximum of a sequence is raised only about log(count) times.  A stale read
// can only cause a needless atomic, never a wrong result.
#ifdef __HIPCC__
__device__ __forceinline__ void fold_absmax(uint32_t *absmax_bits, float mx)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if ((threadIdx.x & 63) == 0) {
        const uint32_t bits = __float_as_uint(mx);
        if (bits > __hip_atomic_load(absmax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(absmax_bits, bits);
    }
}
#endif

}  // namespace dybit
