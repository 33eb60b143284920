// Host check of the launch-constant division the kernels use for the tile walk: for every divisor in a
// dense low range and a spread of large ones, the quotient agrees with the C++ division at the boundaries
// of every quotient step that fits, at both ends of the range, and on a pseudo-random sample.
#include <cstdint>
#include <cstdio>
#include <initializer_list>

#include "fast_div.hpp"

int main()
{
    using gemmf32::FastDiv;
    uint64_t state = 0x9E3779B97F4A7C15ull;
    auto next = [&]() {
        state ^= state << 13; state ^= state >> 7; state ^= state << 17;
        return state;
    };
    long long checked = 0;
    auto check = [&](unsigned d, int64_t n) {
        if (n < 0 || n > 2147483647LL) return true;
        const FastDiv f = gemmf32::make_fast_div(d);
        ++checked;
        if (gemmf32::fast_div_reference((int)n, f) == (int)(n / d)) return true;
        std::printf("FAIL d=%u n=%lld got %d want %lld\n", d, (long long)n, gemmf32::fast_div_reference((int)n, f), (long long)(n / d));
        return false;
    };
    auto check_divisor = [&](unsigned d) {
        const int64_t top = 2147483647LL;
        for (int64_t n : std::initializer_list<int64_t>{0, 1, (int64_t)d - 1, (int64_t)d, (int64_t)d + 1, top - 1, top, top / d * d, top / d * d - 1})
            if (!check(d, n)) return false;
        for (int i = 0; i < 64; ++i) {
            const int64_t q = (int64_t)(next() % (uint64_t)(top / d + 1));
            for (int64_t n : std::initializer_list<int64_t>{q * d - 1, q * d, q * d + d - 1})
                if (!check(d, n)) return false;
            if (!check(d, (int64_t)(next() & 0x7FFFFFFF))) return false;
        }
        return true;
    };
    for (unsigned d = 1; d <= 70000; ++d)
        if (!check_divisor(d)) return 1;
    for (int i = 0; i < 200000; ++i)
        if (!check_divisor((unsigned)(next() % 2147483647ull) + 1)) return 1;
    for (unsigned s = 1; s < 31; ++s)
        for (int delta = -2; delta <= 2; ++delta)
            if ((1u << s) + delta >= 1 && !check_divisor((1u << s) + delta)) return 1;
    std::printf("ok %lld\n", checked);
    return 0;
}
