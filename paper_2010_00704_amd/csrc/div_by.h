// Division by a divisor that is fixed when a kernel is launched.  Plain C++ on purpose: the host
// fills the constants, the device applies them, and a host-only test checks the pair.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define BCNN_HOST_DEVICE __host__ __device__
#else
#define BCNN_HOST_DEVICE
#endif

namespace bcnn {

// floor(n / d) for 0 <= n < 2^31: with s = ceil(log2 d) and mul = floor(2^(31+s) / d) + 1 (which fits
// 32 bits), floor(n / d) = (n * mul) >> (31 + s) exactly, because the error
// n * (mul * d - 2^(31+s)) / (d * 2^(31+s)) stays below 1 / d.  Three instructions (multiply-high, shift,
// select) instead of the thirty of a division by an unknown; d = 1 has no 32-bit multiplier and is selected.
struct DivBy {
    uint32_t mul;
    int32_t shift;   // s - 1
    int32_t d;
    static DivBy make(int32_t d)
    {
        DivBy r{0u, 0, d};
        if (d > 1) {
            int s = 0;
            while ((int64_t(1) << s) < d) ++s;
            r.mul = (uint32_t)((uint64_t(1) << (31 + s)) / (uint64_t)d + 1u);
            r.shift = s - 1;
        }
        return r;
    }
    BCNN_HOST_DEVICE int operator()(int n) const
    {
        const uint32_t hi = (uint32_t)(((uint64_t)(uint32_t)n * (uint64_t)mul) >> 32);
        return d == 1 ? n : (int)(hi >> shift);
    }
};

}  // namespace bcnn
