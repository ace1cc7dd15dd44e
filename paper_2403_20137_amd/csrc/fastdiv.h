// Division of a 31-bit numerator by a run-time constant through one multiply and one shift
// (internal; host and device).  Used where a kernel turns a flat row index into (batch, head, token).
#pragma once

#include <cstdint>

#if defined(__HIPCC__)
#define KVBFP_HD __host__ __device__
#else
#define KVBFP_HD
#endif

namespace kvbfp {

// n / d = (n * mul) >> shift for every 0 <= n < 2^31: with l = ceil(log2 d) and mul = floor(2^(31+l) / d) + 1
// the error of mul * d against 2^(31+l) is at most d <= 2^l, which 31 numerator bits cannot carry into
// the quotient.  mul fits 32 bits.
struct FastDiv { uint32_t mul, shift; };

inline FastDiv make_fastdiv(uint32_t d) {   // d >= 1
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    return FastDiv{(uint32_t)(((1ull << (31 + l)) / d) + 1), 31 + l};
}

KVBFP_HD inline uint32_t fastdiv(uint32_t n, FastDiv d) {
    return (uint32_t)(((uint64_t)n * d.mul) >> d.shift);
}

}  // namespace kvbfp
