// Host build of the GPU library's packed-byte trim (its intrinsics emulated), so the
// bit manipulation can be compared with the oracle over the whole input domain
// without a GPU.  Compiled on the fly by tests/test_swar_host.py.
#include "../paper_2105_11010_amd/csrc/sparq_swar.h"

// out[4 * (a * 256 + b) + i] = byte i of trim4({a, b, b, a}) -- pairs (a,b) and (b,a).
extern "C" void swar_all_pairs(int n, unsigned S, int round_nearest, int pair, unsigned char* out) {
    const sparq::TrimLuts L = sparq::make_luts(n, S);
    for (unsigned a = 0; a < 256; ++a)
        for (unsigned b = 0; b < 256; ++b) {
            const uint32_t x = a | (b << 8) | (b << 16) | (a << 24);
            const uint32_t y = sparq::trim4_any(x, L, round_nearest != 0, pair != 0);
            for (int i = 0; i < 4; ++i) out[4 * (a * 256 + b) + i] = (unsigned char)(y >> (8 * i));
        }
}
