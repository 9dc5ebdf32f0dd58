// Host check of sparq_fastdiv.h: floor(n / d) for dividends below 2^31 against plain division, on every small
// divisor, divisors around powers of two, large and random divisors, and dividends around every multiple that
// could round the wrong way.  Prints "ok <cases>".
#include <stdio.h>
#include <stdint.h>
#include <stdlib.h>
#include <initializer_list>

#include "../paper_2105_11010_amd/csrc/sparq_fastdiv.h"

using namespace sparq;

static long long cases = 0;
static int check(uint32_t n, uint32_t d, const FastDiv& f) {
    ++cases;
    if (fastdiv(n, f) != n / d) { printf("FAIL %u / %u = %u, got %u\n", n, d, n / d, fastdiv(n, f)); return 1; }
    return 0;
}
static int check_divisor(uint32_t d) {
    const FastDiv f = make_fastdiv(d);
    const uint32_t top = 0x7FFFFFFFu;
    const uint32_t fixed[] = {0u, 1u, 2u, d - 1, d, d + 1, 2 * d - 1, 2 * d, top, top - 1, top / 2, top / d * d, top / d * d - 1};
    for (uint32_t n : fixed)
        if (n <= top && check(n, d, f)) return 1;
    for (int i = 0; i < 64; ++i) {
        const uint32_t k = (uint32_t)rand() % (top / d + 1);
        const uint64_t base = (uint64_t)k * d;
        for (int o = -1; o <= 1; ++o) {
            const int64_t n = (int64_t)base + o;
            if (n >= 0 && n <= top && check((uint32_t)n, d, f)) return 1;
        }
        if (check((uint32_t)(((uint32_t)rand() << 16 ^ (uint32_t)rand()) & top), d, f)) return 1;
    }
    return 0;
}
int main() {
    srand(11);
    for (uint32_t d = 1; d <= 70000; ++d)
        if (check_divisor(d)) return 1;
    for (int s = 1; s < 31; ++s)
        for (int o = -2; o <= 2; ++o) {
            const int64_t d = (1ll << s) + o;
            if (d >= 1 && d <= 0x7FFFFFFF && check_divisor((uint32_t)d)) return 1;
        }
    for (int i = 0; i < 20000; ++i) {
        const uint32_t d = (((uint32_t)rand() << 16) ^ (uint32_t)rand()) & 0x7FFFFFFFu;
        if (d >= 1 && check_divisor(d)) return 1;
    }
    // every dividend for a few divisors of the workloads' output sizes
    for (uint32_t d : {7u, 14u, 28u, 35u, 56u, 112u}) {
        const FastDiv f = make_fastdiv(d);
        for (uint32_t n = 0; n < (1u << 24); ++n)
            if (check(n, d, f)) return 1;
    }
    printf("ok %lld\n", cases);
    return 0;
}
