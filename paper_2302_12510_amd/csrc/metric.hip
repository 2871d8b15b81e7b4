// Quantization error of a tensor in a DyBit format (Sec. III-C, Eq. 2) for gfx950: one pass over the
// fp32 tensor, bound by HBM bandwidth (4 bytes per element, nothing written but four doubles).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dybit_device.h"
#include "dybit_host.h"

namespace dybit {
namespace {

constexpr int kThreads = 256;
constexpr int kInFlight = 4;                       // 128-bit loads in flight per lane
typedef float f32x4 __attribute__((ext_vector_type(4)));

// x - x_hat for one element, x_hat = s * (the format's value nearest to |x| / s, saturated).
//
// The error does not depend on which neighbour a tie goes to, and an element within rounding of a
// decision point has (to that rounding) the same error on either side, so no exact decision is
// needed here, unlike in the encoder.  q = |x| * fl(1/s).  Below 1 the values are the multiples of
// 2^-(M-1): a magic-number addition rounds q * 2^(M-1) to an integer.  From 1 up, subtracting q's
// bit pattern from a constant gives 2^M - c(q), c the real-valued code, which is linear between
// neighbouring values (see magnitude_value for the constant); it is rounded to an integer the same
// way and taken back through the same subtraction, which is its own inverse.
template <int M, bool SIGNED>
__device__ __forceinline__ float quant_error(float x, float rinv, float s)
{
    constexpr float vmax = (float)(1u << (M - 1));
    constexpr uint32_t kRecip = (uint32_t)(254 + M - 1) << 23;
    const float kMagic = __uint_as_float(0x4B400000u);                   // 1.5 * 2^23: rounds to an integer
    const float inv_grid = __uint_as_float((uint32_t)(127 - (M - 1)) << 23);
    const float t = SIGNED ? fabsf(x) : fmaxf(x, 0.0f);
    const float q = fminf(t * rinv, vmax);
    const float lin = (fmaf(q, vmax, kMagic) - kMagic) * inv_grid;
    const float n = (__uint_as_float(kRecip - __float_as_uint(q)) + kMagic) - kMagic;
    const float rec = __uint_as_float(kRecip - __float_as_uint(n));
    return fmaf(-s, q < 1.0f ? lin : rec, SIGNED ? fabsf(x) : x);        // one rounding
}

struct Sums {
    double dd, x, xx;
};

template <int M, bool SIGNED>
__device__ __forceinline__ void add4(Sums &a, f32x4 v, float rinv, float s)
{
    const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        // squares and sums in double: d^2 leaves the float range for scales beyond 2^+-60, and the
        // variance is a difference of two sums
        const double d = (double)quant_error<M, SIGNED>(e[k], rinv, s);
        const double xd = (double)e[k];
        a.dd = fma(d, d, a.dd);
        a.x += xd;
        a.xx = fma(xd, xd, a.xx);
    }
}

__global__ void rmse_init_kernel(double *out) { out[1] = out[2] = out[3] = 0.0; }

template <int M, bool SIGNED>
__global__ __launch_bounds__(kThreads) void rmse_kernel(const float *__restrict__ x, size_t n, const float *__restrict__ scale,
                                                        double *__restrict__ out, int *async_error)
{
    const float s = *scale;
    const uint32_t e = (__float_as_uint(s) >> 23) & 0xffu;
    const bool ok = s > 0.0f && e >= 27u && e <= 227u;
    const float rinv = 1.0f / s;
    const size_t n4 = n >> 2;
    const f32x4 *x4 = reinterpret_cast<const f32x4 *>(x);
    Sums a{0.0, 0.0, 0.0};
    // a workgroup reads contiguous chunks of kInFlight x kThreads 128-bit words (loads a whole grid
    // apart, a large power of two, would keep hitting the same memory channels)
    constexpr size_t per_block = (size_t)kThreads * kInFlight;
    for (size_t base = (size_t)blockIdx.x * per_block; base < n4; base += (size_t)gridDim.x * per_block) {
        const size_t i = base + threadIdx.x;
        f32x4 v[kInFlight];
        if (base + per_block <= n4) {                                  // uniform: a whole chunk
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) v[u] = __builtin_nontemporal_load(x4 + i + u * kThreads);
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) add4<M, SIGNED>(a, v[u], rinv, s);
        } else {
            for (int u = 0; u < kInFlight; ++u)
                if (i + u * kThreads < n4) add4<M, SIGNED>(a, x4[i + u * kThreads], rinv, s);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const float xe = x[(n4 << 2) + threadIdx.x];
        const float d = quant_error<M, SIGNED>(xe, rinv, s);
        a.dd += (double)d * (double)d;
        a.x += (double)xe;
        a.xx = fma((double)xe, (double)xe, a.xx);
    }
    // wave, then workgroup, then one atomic per sum and workgroup
    for (int off = 32; off > 0; off >>= 1) {
        a.dd += __shfl_xor(a.dd, off);
        a.x += __shfl_xor(a.x, off);
        a.xx += __shfl_xor(a.xx, off);
    }
    __shared__ double part[kThreads / 64][3];
    if ((threadIdx.x & 63) == 0) {
        part[threadIdx.x >> 6][0] = a.dd;
        part[threadIdx.x >> 6][1] = a.x;
        part[threadIdx.x >> 6][2] = a.xx;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) t += part[w][threadIdx.x];
        if (!ok) t = __builtin_nan("");
        atomicAdd(out + 1 + threadIdx.x, t);
    }
    if (!ok && blockIdx.x == 0 && threadIdx.x == 0) *async_error = DYBIT_ERR_BAD_SCALE;
}

// RMSE = sqrt( (sum d^2 / n) / variance ), variance = sum x^2 / n - (sum x / n)^2.
__global__ void rmse_finish_kernel(double *out, double n)
{
    const double mean = out[2] / n;
    const double var = out[3] / n - mean * mean;
    out[0] = sqrt((out[1] / n) / var);
}

template <int M, bool SIGNED>
void launch_rmse(const float *x, size_t n, const float *scale, double *out, int *flag, hipStream_t st)
{
    size_t blocks = (n / 4 + (size_t)kThreads * kInFlight) / ((size_t)kThreads * kInFlight);
    if (blocks > 256 * 4) blocks = 256 * 4;
    hipLaunchKernelGGL((rmse_kernel<M, SIGNED>), dim3((unsigned)blocks), dim3(kThreads), 0, st, x, n, scale, out, flag);
}

}  // namespace
}  // namespace dybit

using namespace dybit;

extern "C" dybit_status dybit_rmse(const float *x, size_t n, dybit_fmt f, const float *scale, double *out, dybit_stream stream)
{
    dybit_status status = check_fmt(f);
    if (status != DYBIT_OK) return status;
    if (!x || !scale || !out) return DYBIT_ERR_NULL;
    if (n == 0) return DYBIT_ERR_INVALID_ARG;
    if (!aligned16(x) || (reinterpret_cast<uintptr_t>(out) & 7u)) return DYBIT_ERR_ALIGNMENT;
    int *flag = async_error_word();
    if (!flag) return DYBIT_ERR_HIP;
    hipStream_t hs = (hipStream_t)stream;
    hipLaunchKernelGGL(rmse_init_kernel, dim3(1), dim3(1), 0, hs, out);
#define DYBIT_R(M, S) launch_rmse<M, S>(x, n, scale, out, flag, hs)
    switch (f.bits * 2 + f.is_signed) {
        case 4: DYBIT_R(2, false); break;   case 5: DYBIT_R(1, true); break;
        case 8: DYBIT_R(4, false); break;   case 9: DYBIT_R(3, true); break;
        case 12: DYBIT_R(6, false); break;  case 13: DYBIT_R(5, true); break;
        case 16: DYBIT_R(8, false); break;  case 17: DYBIT_R(7, true); break;
    }
#undef DYBIT_R
    hipLaunchKernelGGL(rmse_finish_kernel, dim3(1), dim3(1), 0, hs, out, (double)n);
    return launch_status();
}
