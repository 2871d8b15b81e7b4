// Host-only entry points of libdybit: the code table of a format, packed sizes, status names.
#include <cmath>

#include "dybit_host.h"

namespace {

// Eq. 1 with the Table I reading, spelled out case by case on the host.
double host_magnitude(unsigned c, int m)
{
    const unsigned top = (1u << m) - 1;
    if (c == 0) return 0.0;
    if (c == top) return std::ldexp(1.0, m - 1);                  // all ones: the maximum, 2^(m-1)
    if (!(c & (1u << (m - 1)))) return std::ldexp((double)c, -(m - 1));   // start bit 0: fraction only
    int ones = 0;
    while (c & (1u << (m - 1 - ones))) ++ones;                    // leading-one count i
    const int k = m - ones - 1;                                   // fraction length
    const unsigned frac = c & ((1u << k) - 1);
    return std::ldexp(1.0 + std::ldexp((double)frac, -k), ones - 1);
}

}  // namespace

extern "C" dybit_status dybit_codebook(dybit_fmt f, float *values_out, int32_t *count_out)
{
    const dybit_status st = dybit::check_fmt(f);
    if (st != DYBIT_OK) return st;
    if (!values_out) return DYBIT_ERR_NULL;
    const int m = f.is_signed ? f.bits - 1 : f.bits;
    for (unsigned c = 0; c < (1u << m); ++c) {
        const float v = (float)host_magnitude(c, m);
        values_out[c] = v;
        if (f.is_signed) values_out[(1u << m) | c] = c ? -v : 0.0f;
    }
    if (count_out) *count_out = 1 << f.bits;
    return DYBIT_OK;
}

extern "C" size_t dybit_packed_bytes(dybit_fmt f, size_t n)
{
    if (dybit::check_fmt(f) != DYBIT_OK) return 0;
    return (n * (size_t)f.bits + 7) / 8;
}

extern "C" const char *dybit_status_string(dybit_status s)
{
    switch (s) {
        case DYBIT_OK: return "ok";
        case DYBIT_ERR_INVALID_ARG: return "invalid argument";
        case DYBIT_ERR_UNSUPPORTED_BITS: return "unsupported bitwidth";
        case DYBIT_ERR_BAD_SCALE: return "scale is not a finite normal positive float";
        case DYBIT_ERR_ALIGNMENT: return "misaligned buffer or packed row";
        case DYBIT_ERR_NULL: return "null pointer";
        case DYBIT_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}
