// Host-side argument checks shared by the C-ABI entry points.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/dybit.h"

namespace dybit {

inline dybit_status check_fmt(dybit_fmt f)
{
    if (f.bits != 2 && f.bits != 4 && f.bits != 6 && f.bits != 8) return DYBIT_ERR_UNSUPPORTED_BITS;
    if (f.is_signed != 0 && f.is_signed != 1) return DYBIT_ERR_INVALID_ARG;
    return DYBIT_OK;
}

// Device word that receives the asynchronous errors of this host thread's calls: the caller's own
// (dybit_set_async_error_word) or the library's flag on the current device; NULL on a HIP failure (quantize.hip).
int *async_error_word();

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// A HIP error that a launch function met before its launch (gemm_dispatch.cpp keeps it per host thread).
void note_hip(hipError_t e);
hipError_t take_hip_error();

inline dybit_status launch_status()
{
    const hipError_t before = take_hip_error(), at_launch = hipGetLastError();
    return (before == hipSuccess && at_launch == hipSuccess) ? DYBIT_OK : DYBIT_ERR_HIP;
}

}  // namespace dybit
