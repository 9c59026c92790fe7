// Division of a 31-bit dividend by a run-time constant with one multiply and one shift.
#pragma once

#include <cstdint>

#if defined(__HIPCC__)
#define TP_HD __host__ __device__
#else
#define TP_HD
#endif

namespace tp {

// For a divisor d >= 1 and any n < 2^31:  n / d == (uint64(n) * mul) >> shift,
// with s = ceil(log2 d), shift = 31 + s, mul = ceil(2^shift / d) (fits 32 bits).
// Proof sketch: mul*d = 2^shift + e with 0 <= e < d <= 2^s, so the error term
// n*e / (d * 2^shift) is below 1/d whenever n < 2^31.
struct FastDiv {
    uint32_t mul = 0;
    uint32_t shift = 0;
    uint32_t divisor = 1;
};

inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.divisor = d;
    uint32_t s = 0;
    while ((uint64_t{1} << s) < d) ++s;
    f.shift = 31 + s;
    const unsigned __int128 one = 1;
    f.mul = static_cast<uint32_t>(((one << f.shift) + d - 1) / d);
    return f;
}

TP_HD inline uint32_t fastdiv(uint32_t n, const FastDiv& f) {
    return static_cast<uint32_t>((static_cast<uint64_t>(n) * f.mul) >> f.shift);
}

}  // namespace tp
