// Division of a 31-bit unsigned number by a divisor known on the host before the launch: one
// multiply-high and a shift on the device instead of the ~30 instructions of an emulated
// 32-bit division.  The work-list arithmetic of the kernels' prologue sits on the latency-critical
// path of every call, which is why this exists.
//
// Plain C++ (also compiled by the host compiler in the CPU tests).
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define FD_HOST_DEVICE __host__ __device__
#else
#define FD_HOST_DEVICE
#endif

namespace fd {

// mul == 0: the divisor is 2^shift.  Otherwise floor(n / d) = mulhi(n, mul) >> shift for every
// n < 2^31 (round-up method: with l = ceil(log2 d), mul = floor(2^(31+l) / d) + 1 satisfies
// 2^(31+l) < mul * d <= 2^(31+l) + 2^l, which makes the truncated product exact; shift = l - 1).
struct FastDiv {
    uint32_t mul, shift;
};

inline FastDiv make_fastdiv(uint32_t d)      // 1 <= d < 2^31
{
    FastDiv f = {0u, 0u};
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;             // l = ceil(log2 d)
    if ((1ull << l) == d) {
        f.shift = l;
        return f;
    }
    f.mul = (uint32_t)(((1ull << (31 + l)) / d) + 1ull);
    f.shift = l - 1;
    return f;
}

FD_HOST_DEVICE inline uint32_t fast_div(uint32_t n, FastDiv f)
{
    const uint32_t hi = (uint32_t)(((uint64_t)n * f.mul) >> 32);
    return (f.mul ? hi : n) >> f.shift;
}

}  // namespace fd
