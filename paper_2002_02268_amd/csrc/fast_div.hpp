// Division of a walk position (0 <= n < 2^31) by a divisor d >= 1 that is fixed for the launch: the host
// works out s = ceil(log2 d) and magic = ceil(2^(31 + s) / d) (below 2^32; exact for every such n because
// magic * d - 2^(31 + s) < d <= 2^s), and the kernel takes the high half of n * magic and shifts: two scalar
// instructions where the division itself is a chain of about 25 at the head of every workgroup.
// Host code only in this file (the kernel header holds the device side), so that it can be checked by itself.
#pragma once
#include <cstdint>

namespace gemmf32 {

struct FastDiv {
    unsigned magic;             // 0 for d == 1
    unsigned shift;             // s - 1
};

inline FastDiv make_fast_div(unsigned d)
{
    if (d <= 1) return FastDiv{0u, 0u};
    unsigned s = 0;
    while ((1ull << s) < d) ++s;
    const unsigned long long m = ((1ull << (31 + s)) + d - 1) / d;
    return FastDiv{(unsigned)m, s - 1};
}

// what the kernel computes, spelled out for the host
inline int fast_div_reference(int n, const FastDiv f)
{
    return f.magic == 0 ? n : (int)((((uint64_t)(unsigned)n * f.magic) >> 32) >> f.shift);
}

}  // namespace gemmf32
