// CPU check of the multiply-shift division the cache-write kernel uses to turn a flat row index into
// (batch, head, token): fastdiv(n, make_fastdiv(d)) == n / d for every numerator below 2^31.
//   - every numerator, for four divisors (small odd, just above a power of two twice, the largest possible);
//   - for every divisor up to 70 000 and a spread of larger ones: the numerators around every multiple of d
//     that a coarse stride reaches, plus both ends of the range (the only places a quotient can go wrong are
//     just below a multiple of d, where the approximation error of the multiplier is largest relative to
//     the distance to the next integer).
#include <cstdint>
#include <cstdio>
#include <cstdlib>

#include "fastdiv.h"

using kvbfp::fastdiv;
using kvbfp::make_fastdiv;

static int check(uint32_t n, uint32_t d, kvbfp::FastDiv f) {
    if (fastdiv(n, f) != n / d) {
        std::printf("FAIL n=%u d=%u got %u want %u\n", n, d, fastdiv(n, f), n / d);
        return 1;
    }
    return 0;
}

int main() {
    const uint32_t kMax = 0x7FFFFFFFu;
    int bad = 0;
    const uint32_t full[] = {3u, 4097u, 32769u, 0x7FFFFFFFu};
    for (uint32_t d : full) {
        const kvbfp::FastDiv f = make_fastdiv(d);
        uint32_t q = 0, r = 0;                       // running n / d and n % d, so the check itself has no division
        for (uint32_t n = 0;; ++n) {
            if (fastdiv(n, f) != q) { std::printf("FAIL n=%u d=%u\n", n, d); ++bad; break; }
            if (n == kMax) break;
            if (++r == d) { r = 0; ++q; }
        }
    }
    auto edges = [&](uint32_t d) {
        const kvbfp::FastDiv f = make_fastdiv(d);
        bad += check(0, d, f) + check(kMax, d, f) + check(kMax - 1, d, f);
        const uint64_t n_mult = (uint64_t)kMax / d;
        const uint64_t step = n_mult / 4096 + 1;
        for (uint64_t k = 1; k <= n_mult; k += step) {
            const uint64_t m = k * d;
            bad += check((uint32_t)(m - 1), d, f) + check((uint32_t)m, d, f);
            if (m + 1 <= kMax) bad += check((uint32_t)(m + 1), d, f);
        }
        const uint64_t last = n_mult * d;          // the largest multiple inside the range
        bad += check((uint32_t)(last - 1), d, f) + check((uint32_t)last, d, f);
    };
    for (uint32_t d = 1; d <= 70000; ++d) edges(d);
    for (uint64_t d = 70001; d <= kMax; d += 104729 + (d >> 7)) edges((uint32_t)d);
    if (bad) { std::printf("%d failures\n", bad); return 1; }
    std::printf("fastdiv ok\n");
    return 0;
}
