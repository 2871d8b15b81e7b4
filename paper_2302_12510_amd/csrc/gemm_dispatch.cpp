// Chooses between the tiled MFMA kernels of the DyBit matrix product.
//
// All need signed weights, K (convolution: Cin) a multiple of 64 (2- and 6-bit operands on the 256 x 256 kernel: of 128) so that
// a 64-wide k group is one run of whole 128-bit loads inside one filter tap, 16-byte aligned
// code buffers, and buffers below 2 GiB (32-bit buffer offsets).  The 256 x 256 kernel does the
// least decode work per MFMA and is used when its tiles can fill the 256 compute units, N is
// wide enough for them and K is long enough for the main loop to outweigh the epilogue; the
// 128 x 128 kernel takes the rest.  dybit_set_option (initial values: the environment, read once)
// overrides the choice whenever the named kernel's preconditions hold; every launch records the kernel
// it started, which dybit_last_gemm_kernel reports, so a test can tell which kernel it exercised.
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>

#include "../../include/dybit.h"
#include "gemm_args.h"

namespace dybit {

namespace {

std::atomic<int> opt_kernel{0}, opt_mfma_f16{0}, opt_mid_tile{0}, opt_mid_kgroups{0}, opt_ws_off{0};
thread_local int last_kernel = DYBIT_KERNEL_NONE;
thread_local hipError_t pending_hip_error = hipSuccess;

// name / value -> option; false for an unknown pair.  "auto" resets an option.
bool apply_option(const char *name, const char *value)
{
    const bool is_auto = !strcmp(value, "auto");
    if (!strcmp(name, "gemm_kernel")) {
        const int v = is_auto ? 0 : !strcmp(value, "general") ? DYBIT_FORCE_GENERAL : !strcmp(value, "mid") ? DYBIT_FORCE_MID
                    : !strcmp(value, "large") ? DYBIT_FORCE_LARGE : !strcmp(value, "ws") ? DYBIT_FORCE_WS : -1;
        if (v < 0) return false;
        opt_kernel = v;
    } else if (!strcmp(name, "gemm_mfma")) {
        if (!is_auto && strcmp(value, "f16")) return false;
        opt_mfma_f16 = is_auto ? 0 : 1;
    } else if (!strcmp(name, "mid_tile")) {
        const int v = is_auto ? 0 : !strcmp(value, "64") ? 64 : !strcmp(value, "128") ? 128 : -1;
        if (v < 0) return false;
        opt_mid_tile = v;
    } else if (!strcmp(name, "mid_kgroups")) {
        const int v = is_auto ? 0 : !strcmp(value, "1") ? 1 : !strcmp(value, "2") ? 2 : -1;
        if (v < 0) return false;
        opt_mid_kgroups = v;
    } else if (!strcmp(name, "gemm_ws")) {
        if (!is_auto && strcmp(value, "off")) return false;
        opt_ws_off = is_auto ? 0 : 1;
    } else {
        return false;
    }
    return true;
}

// The environment gives the initial values, once; values it cannot hold are ignored.
void options_from_environment()
{
    static const bool done = [] {
        static const char *const vars[][2] = {{"DYBIT_GEMM_KERNEL", "gemm_kernel"}, {"DYBIT_GEMM_MFMA", "gemm_mfma"},
                                              {"DYBIT_MID_TILE", "mid_tile"}, {"DYBIT_MID_KGROUPS", "mid_kgroups"}};
        for (const auto &v : vars) {
            const char *e = getenv(v[0]);
            if (e && *e) apply_option(v[1], e);
        }
        const char *ws = getenv("DYBIT_GEMM_WS");
        if (ws && !strcmp(ws, "0")) apply_option("gemm_ws", "off");
        return true;
    }();
    (void)done;
}

}  // namespace

DispatchOptions dispatch_options()
{
    options_from_environment();
    return DispatchOptions{opt_kernel.load(), opt_mfma_f16.load(), opt_mid_tile.load(), opt_mid_kgroups.load(), opt_ws_off.load()};
}

void note_kernel(int id) { last_kernel = id; }
void note_hip(hipError_t e)
{
    if (e != hipSuccess && pending_hip_error == hipSuccess) pending_hip_error = e;
}
void clear_call_record()
{
    last_kernel = DYBIT_KERNEL_NONE;
    pending_hip_error = hipSuccess;
}
hipError_t take_hip_error()
{
    const hipError_t e = pending_hip_error;
    pending_hip_error = hipSuccess;
    return e;
}

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
    const bool dense = conv && (int64_t)g.pix_bytes * 8 == (int64_t)g.Cin * a_bits;   // not one channel group of a wider image
    const bool rows = dense && g.Cin < 64 && (int64_t)g.kw * g.Cin == 32 && g.a_bytes % 4 == 0;   // fetched as aligned words: none may reach past the tensor
    if (conv && g.Cin % 64 && !rows) return false;
    if ((reinterpret_cast<uintptr_t>(g.A) | reinterpret_cast<uintptr_t>(g.W)) & 15) return false;
    if (g.a_bytes >= 0x7fffffff || g.w_bytes >= 0x7fffffff) return false;

    bool large;
    const bool low_pair = (a_bits == 4 || a_bits == 2) && (w_bits == 4 || w_bits == 2);
    const DispatchOptions opt = dispatch_options();
    const int force = opt.kernel;
    if (force == DYBIT_FORCE_GENERAL) return false;

    // Weight-stationary kernel: the decoded weights of up to 128 columns (N > 128: of a group of 64) stay in
    // LDS, for many rows against few weights (it declines when the weights do not fit).  Wider than 128 columns
    // it is taken where it was measured faster than the 128 x 128 kernel (M x N x K from 401408 x 256 x 64 to
    // 25088 x 1024 x 256): with the write-back epilogue and a short K, 1.05 to 1.25 times; with fp32 results
    // only its 256-byte row segments lose to the tile's 512-byte ones.
    const bool ws_wide = g.q_out != nullptr && g.K <= 256 && (g.C == nullptr || g.K >= 128);
    if (force == DYBIT_FORCE_WS || (!force && !opt.ws_off && g.M >= 16384 && (g.N <= 128 || ws_wide))) {
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
    if (force == DYBIT_FORCE_LARGE) {
        large = true;
    } else if (force == DYBIT_FORCE_MID) {
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
    // fp16 rate, byte decoders) takes them unless the "gemm_mfma" option asks for the fp16 kernels
    const bool wb = g.q_out != nullptr;                             // write-back builds of the same kernels
    if (low_pair && !rows && !opt.mfma_f16) {
        if (w_bits == 4) return (wb ? launch_gemm_f8_w0_wb : launch_gemm_f8_w0)(g, a_bits, conv, large, st);
        return (wb ? launch_gemm_f8_w6_wb : launch_gemm_f8_w6)(g, a_bits, conv, large, st);
    }
    if (rows) large = false;
    if (large) {                                                   // declines a 2- or 6-bit operand unless K (Cin) is a multiple of 128
        bool done;
        if (w_bits == 4) done = (wb ? launch_gemm_fast_w0_wb : launch_gemm_fast_w0)(g, a_bits, conv, st);
        else if (w_bits == 6) done = (wb ? launch_gemm_fast_w4_wb : launch_gemm_fast_w4)(g, a_bits, conv, st);
        else if (w_bits == 2) done = (wb ? launch_gemm_fast_w6_wb : launch_gemm_fast_w6)(g, a_bits, conv, st);
        else done = (wb ? launch_gemm_fast_w2_wb : launch_gemm_fast_w2)(g, a_bits, conv, st);
        if (done) return true;
    }
    if (w_bits == 4) return (wb ? launch_gemm_mid_w0_wb : launch_gemm_mid_w0)(g, a_bits, conv, st);
    if (w_bits == 6) return (wb ? launch_gemm_mid_w4_wb : launch_gemm_mid_w4)(g, a_bits, conv, st);
    if (w_bits == 2) return (wb ? launch_gemm_mid_w6_wb : launch_gemm_mid_w6)(g, a_bits, conv, st);
    return (wb ? launch_gemm_mid_w2_wb : launch_gemm_mid_w2)(g, a_bits, conv, st);
}

}  // namespace dybit

extern "C" int32_t dybit_last_gemm_kernel(void) { return dybit::last_kernel; }

extern "C" dybit_status dybit_set_option(const char *name, const char *value)
{
    if (!name || !value) return DYBIT_ERR_NULL;
    dybit::options_from_environment();                              // so that a later first use does not overwrite this
    return dybit::apply_option(name, value) ? DYBIT_OK : DYBIT_ERR_INVALID_ARG;
}
