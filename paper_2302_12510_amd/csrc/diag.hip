// Measurement aid: the rate of the fp16 matrix cores alone on this device, with operand values
// supplied by the caller (the sustained clock of an MFMA-bound kernel depends on how much the
// operand bits toggle, so the benchmark feeds it decoded DyBit values of the workload).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dybit_host.h"

namespace dybit {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// 8 waves per workgroup, 8 independent 32x32 accumulators per wave, operands held in registers.
__global__ __launch_bounds__(512) void mfma_only_kernel(const f16x8 *__restrict__ operands, int iters, float *sink)
{
    const f16x8 a = operands[threadIdx.x];
    f16x8 b[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) b[j] = operands[512 * (1 + j) + threadIdx.x];
    f32x16 c[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) c[j][v] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b[j], c[j], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += c[j][v];
    if (s == 1.2345e-30f) sink[0] = s;   // keeps the accumulators alive; practically never taken
}

typedef int i32x8 __attribute__((ext_vector_type(8)));

// The same for the fp8 (e4m3) instruction of the 4-bit pairs: operands are bytes, 32 per lane.
__global__ __launch_bounds__(512) void mfma_only_f8_kernel(const i32x8 *__restrict__ operands, int iters, float *sink)
{
    const i32x8 a = operands[threadIdx.x];
    i32x8 b[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) b[j] = operands[512 * (1 + j) + threadIdx.x];
    f32x16 c[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) c[j][v] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) c[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b[j], c[j], 0, 0, 0, 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += c[j][v];
    if (s == 1.2345e-30f) sink[0] = s;
}

}  // namespace dybit

extern "C" dybit_status dybit_diag_mfma_f8(const void *operands, int32_t workgroups, int32_t iters,
                                           float *sink, double *flops_out, dybit_stream stream)
{
    if (!operands || !sink) return DYBIT_ERR_NULL;
    if (workgroups < 1 || iters < 1 || !dybit::aligned16(operands)) return DYBIT_ERR_INVALID_ARG;
    hipLaunchKernelGGL(dybit::mfma_only_f8_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)stream,
                       reinterpret_cast<const dybit::i32x8 *>(operands), iters, sink);
    if (flops_out) *flops_out = (double)workgroups * 8.0 * iters * 8.0 * (2.0 * 32 * 32 * 64);
    return dybit::launch_status();
}

extern "C" dybit_status dybit_diag_mfma_f16(const void *operands, int32_t workgroups, int32_t iters,
                                            float *sink, double *flops_out, dybit_stream stream)
{
    if (!operands || !sink) return DYBIT_ERR_NULL;
    if (workgroups < 1 || iters < 1 || !dybit::aligned16(operands)) return DYBIT_ERR_INVALID_ARG;
    hipLaunchKernelGGL(dybit::mfma_only_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)stream,
                       reinterpret_cast<const dybit::f16x8 *>(operands), iters, sink);
    if (flops_out) *flops_out = (double)workgroups * 8.0 * iters * 8.0 * (2.0 * 32 * 32 * 16);
    return dybit::launch_status();
}
