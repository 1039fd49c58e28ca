// Host-only check of the launch-time division constants (csrc/div_by.h) against the C++ division:
// every divisor up to 70 000 on edge values and a spread of dividends, the largest divisors, and both
// neighbours of every multiple below 2^31 for the divisors the benchmark shapes use and 300 others.  Exit status 0 = all equal.
#include "div_by.h"

#include <cstdio>
#include <initializer_list>

int main()
{
    using bcnn::DivBy;
    long bad = 0;
    const int64_t top = (int64_t(1) << 31) - 1;
    for (int d = 1; d <= 70000; ++d) {
        const DivBy f = DivBy::make(d);
        const int64_t pts[] = {0, 1, d - 1, d, d + 1, 2LL * d - 1, 2LL * d, 1000003, top, top + 1 - d, int64_t(1) << 30,
                               top / d * d, top / d * d - 1};
        for (int64_t n : pts)
            if (n >= 0 && n <= top && f((int)n) != (int)(n / d)) ++bad;
        for (int64_t i = 0; i < 2000; ++i) {
            const int64_t n = (i * 715827883LL + d * 7919LL) % (top + 1);
            if (f((int)n) != (int)(n / d)) ++bad;
        }
    }
    for (int d : {2147483647, 1073741824, 1073741825, 536870913, 100000007})
        for (int64_t n : {int64_t(0), int64_t(d) - 1, int64_t(d), top})
            if (DivBy::make(d)((int)n) != (int)(n / d)) ++bad;
    // a wrong quotient shows first next to a multiple of d: every q * d - 1 and q * d below 2^31, for the
    // divisors of the benchmark shapes and a few hundred others
    auto boundaries = [&](int d) {
        const DivBy f = DivBy::make(d);
        for (int64_t q = 0; q * d <= top; ++q) {
            const int64_t n = q * d;
            if (f((int)n) != (int)q) { ++bad; return; }
            if (n > 0 && f((int)(n - 1)) != (int)(q - 1)) { ++bad; return; }
        }
    };
    for (int d : {49, 196, 784, 3136, 7, 14, 28, 56, 641}) boundaries(d);
    for (int i = 0; i < 300; ++i) boundaries(1000 + 37 * i * i + i);
    for (int n = 0; n < (1 << 24); ++n)
        if (DivBy::make(49)(n) != n / 49 || DivBy::make(3)(n) != n / 3) { ++bad; break; }
    std::printf("mismatches: %ld\n", bad);
    return bad != 0;
}
