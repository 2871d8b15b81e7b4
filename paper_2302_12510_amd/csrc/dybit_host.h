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

// Device address of the asynchronous error flag of the current device, or NULL (quantize.hip).
int *async_error_word();

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline dybit_status launch_status()
{
    return hipGetLastError() == hipSuccess ? DYBIT_OK : DYBIT_ERR_HIP;
}

}  // namespace dybit
