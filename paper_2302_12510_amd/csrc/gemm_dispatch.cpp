// Chooses between the tiled MFMA kernels of the DyBit matrix product.
//
// All need signed weights (2- and 6-bit operands: the 128 x 128 fp16 kernel only), K (convolution: Cin) a multiple of 64 so that
// a 64-wide k group is one run of whole 128-bit loads inside one filter tap, 16-byte aligned
// code buffers, and buffers below 2 GiB (32-bit buffer offsets).  The 256 x 256 kernel does the
// least decode work per MFMA and is used when its tiles can fill the 256 compute units, N is
// wide enough for them and K is long enough for the main loop to outweigh the epilogue; the
// 128 x 128 kernel takes the rest.  The environment variable
// DYBIT_GEMM_KERNEL = large | mid | general overrides the choice whenever the named kernel's
// preconditions hold (tests use it to reach a given kernel with small shapes); DYBIT_GEMM_MFMA=f16
// keeps pairs of 4-bit operands on the fp16 kernels instead of the fp8 ones.
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include "gemm_args.h"

namespace dybit {

void launch_gemm_general_wb(const GemmArgs &g, int a_bits, int w_bits, bool conv, int mode, hipStream_t st)
{
    switch (a_bits) {
        case 2: launch_gemm_general_a2_wb(g, w_bits, conv, mode, st); break;
        case 4: launch_gemm_general_a4_wb(g, w_bits, conv, mode, st); break;
        case 6: launch_gemm_general_a6_wb(g, w_bits, conv, mode, st); break;
        case 8: launch_gemm_general_a8_wb(g, w_bits, conv, mode, st); break;
    }
}

bool launch_gemm_tiled(const GemmArgs &g, int a_bits, int w_bits, bool conv, hipStream_t st)
{
    if (!g.w_signed) return false;                                  // every width 2, 4, 6, 8 has a decoder; weights are signed
    if (g.M < 1 || g.N < 1 || g.K < 64 || g.K % 64) return false;
    // a convolution needs whole 64-code k groups inside a filter tap, or (few channels) filter rows of
    // exactly 32 codes, which the 128 x 128 kernel fetches row by row
    const bool rows = conv && g.Cin < 64 && (int64_t)g.kw * g.Cin == 32;
    if (conv && g.Cin % 64 && !rows) return false;
    if ((reinterpret_cast<uintptr_t>(g.A) | reinterpret_cast<uintptr_t>(g.W)) & 15) return false;
    if (g.a_bytes >= 0x7fffffff || g.w_bytes >= 0x7fffffff) return false;

    bool large;
    const bool low_pair = (a_bits == 4 || a_bits == 2) && (w_bits == 4 || w_bits == 2);
    const char *force = getenv("DYBIT_GEMM_KERNEL");
    if (force && !strcmp(force, "general")) return false;

    // Weight-stationary kernel: the whole decoded weight matrix in LDS, for many rows against few
    // weights (it declines when the weights do not fit).  DYBIT_GEMM_KERNEL=ws forces it where it fits.
    const bool ws_forced = force && !strcmp(force, "ws");
    const char *ws_env = getenv("DYBIT_GEMM_WS");                  // DYBIT_GEMM_WS=0 keeps it out of the automatic choice
    const bool ws_off = ws_env && !strcmp(ws_env, "0");
    if (ws_forced || (!force && !ws_off && g.N <= 128 && g.M >= 16384)) {
        const bool wb_ = g.q_out != nullptr;
        bool done = false;
        switch (w_bits) {
            case 4: done = (wb_ ? launch_gemm_ws_w0_wb : launch_gemm_ws_w0)(g, a_bits, conv, st); break;
            case 8: done = (wb_ ? launch_gemm_ws_w2_wb : launch_gemm_ws_w2)(g, a_bits, conv, st); break;
            case 6: done = (wb_ ? launch_gemm_ws_w4_wb : launch_gemm_ws_w4)(g, a_bits, conv, st); break;
            case 2: done = (wb_ ? launch_gemm_ws_w6_wb : launch_gemm_ws_w6)(g, a_bits, conv, st); break;
        }
        if (done) return true;
    }
    if (force && !strcmp(force, "large")) {
        large = true;
    } else if (force && !strcmp(force, "mid")) {
        large = false;
    } else {
        // Too few 256 x 256 tiles cannot fill 256 compute units, and a narrow N wastes most of a
        // 256-wide tile.  With a short K the epilogue (the stores of C, the loads of the shortcut)
        // dominates, and the 128 x 128 kernel with three workgroups per compute unit keeps more
        // of those memory operations in flight: measured over M x N from 6272 x 2048 to
        // 401408 x 256, it is 1.1 to 1.7 times faster up to K = 512, level at K = 1024 (fp16
        // kernels) or K = 2048 (fp8 kernels), and 10 to 30 % slower beyond.
        const int64_t tiles256 = ((g.M + 255) / 256) * ((g.N + 255) / 256);
        large = g.N > 128 && tiles256 >= 128 && g.K >= (low_pair ? 2048 : 1024);
    }
    // two operands of 4 or 2 bits: every value is exact in e4m3, so the fp8 matrix path (twice the
    // fp16 rate, byte decoders) takes them unless DYBIT_GEMM_MFMA=f16 asks for the fp16 kernels
    const char *mfma = getenv("DYBIT_GEMM_MFMA");
    const bool wb = g.q_out != nullptr;                             // write-back builds of the same kernels
    if (low_pair && !rows && !(mfma && !strcmp(mfma, "f16"))) {
        if (w_bits == 4) return (wb ? launch_gemm_f8_w0_wb : launch_gemm_f8_w0)(g, a_bits, conv, large, st);
        return (wb ? launch_gemm_f8_w6_wb : launch_gemm_f8_w6)(g, a_bits, conv, large, st);
    }
    const bool mid_only = (a_bits != 4 && a_bits != 8) || (w_bits != 4 && w_bits != 8);   // fp16 kernels, 2- and 6-bit operands: the 128 x 128 kernel only
    if (mid_only || rows) large = false;
    if (large) {
        if (w_bits == 4) return (wb ? launch_gemm_fast_w0_wb : launch_gemm_fast_w0)(g, a_bits, conv, st);
        return (wb ? launch_gemm_fast_w2_wb : launch_gemm_fast_w2)(g, a_bits, conv, st);
    }
    if (w_bits == 4) return (wb ? launch_gemm_mid_w0_wb : launch_gemm_mid_w0)(g, a_bits, conv, st);
    if (w_bits == 6) return (wb ? launch_gemm_mid_w4_wb : launch_gemm_mid_w4)(g, a_bits, conv, st);
    if (w_bits == 2) return (wb ? launch_gemm_mid_w6_wb : launch_gemm_mid_w6)(g, a_bits, conv, st);
    return (wb ? launch_gemm_mid_w2_wb : launch_gemm_mid_w2)(g, a_bits, conv, st);
}

}  // namespace dybit
