// Division of a dividend below 2^31 by a divisor that is fixed per launch: one multiply-high and one shift
// instead of the compiler's 64-bit division sequence (hundreds of instructions per output pixel's coordinates).
//
// For d >= 2 let s = ceil(log2 d) - 1, so that 2^s < d <= 2^(s+1), and mul = ceil(2^(32+s) / d), which lies in
// [2^31, 2^32).  Then mul * d = 2^(32+s) + e with 0 <= e < d <= 2^(s+1), and for n < 2^31
//   n * mul / 2^(32+s) = n / d + n * e / (d * 2^(32+s)),   the second term < 2^31 * 2^(s+1) / (d * 2^(32+s)) = 1 / d,
// too small to carry the quotient over the next integer: floor(n * mul / 2^(32+s)) = floor(n / d).
// The file compiles for the host as well; tests/fastdiv_check.cpp checks it against plain division.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define SPARQ_FD __host__ __device__ __forceinline__
#else
#define SPARQ_FD inline
#endif

namespace sparq {

struct FastDiv {
    uint32_t mul, shift;
    uint32_t one;            // the divisor is 1: the quotient is the dividend
};

inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f{0u, 0u, 1u};
    if (d <= 1) return f;
    uint32_t s = 0;
    while ((1ull << (s + 1)) < d) ++s;                       // 2^s < d <= 2^(s+1)
    f.mul = (uint32_t)(((1ull << (32 + s)) + d - 1) / d);
    f.shift = s;
    f.one = 0;
    return f;
}

// floor(n / d) for n < 2^31
SPARQ_FD uint32_t fastdiv(uint32_t n, const FastDiv& f) {
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t hi = __umulhi(n, f.mul);
#else
    const uint32_t hi = (uint32_t)(((uint64_t)n * f.mul) >> 32);
#endif
    return f.one ? n : hi >> f.shift;
}

}  // namespace sparq
