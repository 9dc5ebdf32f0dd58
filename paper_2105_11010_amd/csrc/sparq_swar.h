// SPARQ activation trim on four packed uint8 values (SIMD within a register).
//
// One 32-bit word holds four consecutive input channels c..c+3 with c a
// multiple of 2, so the two vSPARQ pairs (Section 3.2, Eq. 2) are bytes (0,1)
// and (2,3).  bSPARQ (Section 3.1) is expressed through one per-byte mask,
// `low` = 2^s - 1, the residual bits below the chosen window [s+n-1 : s]:
//
//   plain trim   : x & ~low
//   round (+R)   : add 2^s when the residual's top bit is set, unless the
//                  window already holds 2^n - 1 (saturation)
//
// `low` only depends on the position p of the leading one.  It is looked up
// with two byte-permute instructions used as 8-entry tables: table A is
// indexed by x >> 5 (resolves p = 5, 6, 7), table B by (x >> 2) & 7 (resolves
// p = 2, 3, 4 when x < 32).  Masks grow with p, so OR-ing a stale table-B
// entry into a table-A result is harmless.  The tables are built on the host
// from (window_bits, shift_mask), which makes every option set -- 5opt, 3opt,
// 2opt, the 3-bit/6opt and 2-bit/7opt variants (Section 5.1) and any other
// valid mask -- run through the same instructions.
//
// Byte-wise predicates (value == 0, window saturated) come from v_lerp_u8,
// whose 9-bit per-byte sum leaves a carry flag in bit 7, expanded to a byte
// mask with the sign-replicating selectors of v_perm_b32.
//
// The file compiles for the host as well (the intrinsics are emulated) so the
// bit manipulation can be checked exhaustively without a GPU.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define SPARQ_HD __host__ __device__ __forceinline__
#else
#define SPARQ_HD inline
#endif

namespace sparq {

// ---- per-launch constants ---------------------------------------------------
struct TrimLuts {
    uint32_t a_lo, a_hi;     // n-bit window:  low mask by (x >> 5)
    uint32_t b_lo, b_hi;     //                low mask by (x >> 2) & 7
    uint32_t wa_lo, wa_hi;   // 2n-bit window (zero partner, n < 4): same two tables
    uint32_t wb_lo, wb_hi;
    uint32_t ncap_lo, ncap_hi; // n = 4 rounding: 256 - (first value that saturates), by (x >> 5); 0 = never
    uint32_t ones_n;         // 2^n  - 1 in every byte
    uint32_t ones_w;         // 2^2n - 1 in every byte
    uint32_t n;              // window bits
    uint32_t n2;             // 2n
};

// Smallest allowed shift whose window reaches bit p; shifts with bit t set in S.
inline int trim_shift_for(int p, int n, uint32_t S) {
    for (int t = 0; t <= 8; ++t)
        if (((S >> t) & 1u) && t + n - 1 >= p) return t;
    return 8;
}

inline void fill_tables(int n, uint32_t S, uint32_t* a_lo, uint32_t* a_hi, uint32_t* b_lo, uint32_t* b_hi) {
    // leading-one position represented by each table index
    static const int pa[8] = {-1, 5, 6, 6, 7, 7, 7, 7};   // index = x >> 5
    static const int pb[8] = {-1, 2, 3, 3, 4, 4, 4, 4};   // index = (x >> 2) & 7, meaningful for x < 32
    uint64_t A = 0, B = 0;
    for (int i = 0; i < 8; ++i) {
        uint64_t la = pa[i] < 0 ? 0 : ((1u << trim_shift_for(pa[i], n, S)) - 1u);
        uint64_t lb = pb[i] < 0 ? 0 : ((1u << trim_shift_for(pb[i], n, S)) - 1u);
        A |= (la & 0xFF) << (8 * i);
        B |= (lb & 0xFF) << (8 * i);
    }
    *a_lo = (uint32_t)A; *a_hi = (uint32_t)(A >> 32);
    *b_lo = (uint32_t)B; *b_hi = (uint32_t)(B >> 32);
}

// Placements of the 2n-bit window a value gets when its partner is zero: the two n-bit multipliers of Eq. 4
// serve it as a high and a low half, so t is a placement when t and t + n both are n-bit placements (and the
// window stays inside the byte: t <= 8 - 2n).
inline uint32_t wide_shift_mask(int n, uint32_t S) {
    return S & (S >> n) & ((2u << (8 - 2 * n)) - 1u);
}

inline TrimLuts make_luts(int n, uint32_t S) {
    TrimLuts L{};
    L.n = (uint32_t)n;
    L.n2 = (uint32_t)(2 * n);
    if (n >= 8) return L;                      // plain 8-bit layer: tables unused
    fill_tables(n, S, &L.a_lo, &L.a_hi, &L.b_lo, &L.b_hi);
    if (2 * n < 8) fill_tables(2 * n, wide_shift_mask(n, S), &L.wa_lo, &L.wa_hi, &L.wb_lo, &L.wb_hi);
    if (n == 4) {
        // A value saturates when its leading one sits at the window top and the window plus
        // the rounding bit are all ones: x >= 2^(p+1) - 2^(s-1).  Index 0 stands for p = 4
        // (smaller values never round up past 15).
        static const int pa[8] = {4, 5, 6, 6, 7, 7, 7, 7};
        uint64_t C = 0;
        for (int i = 0; i < 8; ++i) {
            const int p = pa[i], sh = trim_shift_for(p, 4, S);
            const uint64_t ncap = (sh >= 1 && p == sh + 3) ? 256u - (1u << (p + 1)) + (1u << (sh - 1)) : 0u;
            C |= (ncap & 0xFF) << (8 * i);
        }
        L.ncap_lo = (uint32_t)C; L.ncap_hi = (uint32_t)(C >> 32);
    }
    L.ones_n = 0x01010101u * ((1u << n) - 1u);
    L.ones_w = 0x01010101u * ((1u << (2 * n > 8 ? 8 : 2 * n)) - 1u);
    return L;
}

// ---- intrinsics (emulated on the host) --------------------------------------
#if defined(__HIP_DEVICE_COMPILE__)
SPARQ_HD uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel) { return __builtin_amdgcn_perm(hi, lo, sel); }
SPARQ_HD uint32_t lerp(uint32_t a, uint32_t b, uint32_t c) { return __builtin_amdgcn_lerp(a, b, c); }
#else
SPARQ_HD uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel) {
    const uint64_t pool = ((uint64_t)hi << 32) | lo;
    uint32_t r = 0;
    for (int i = 0; i < 4; ++i) {
        const uint32_t s = (sel >> (8 * i)) & 0xFF;
        uint32_t b;
        if (s >= 13) b = 0xFF;
        else if (s == 12) b = 0x00;
        else if (s >= 8) b = ((pool >> (8 * (2 * (s - 8) + 1) + 7)) & 1) ? 0xFF : 0x00;
        else b = (uint32_t)(pool >> (8 * s)) & 0xFF;
        r |= b << (8 * i);
    }
    return r;
}
SPARQ_HD uint32_t lerp(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t r = 0;
    for (int i = 0; i < 4; ++i) {
        const uint32_t s = ((a >> (8 * i)) & 0xFF) + ((b >> (8 * i)) & 0xFF) + ((c >> (8 * i)) & 1);
        r |= ((s >> 1) & 0xFF) << (8 * i);
    }
    return r;
}
#endif

SPARQ_HD uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (mask & a) | (~mask & b); }

// 0xFF in every byte whose bit 7 is set in f
SPARQ_HD uint32_t expand_bit7(uint32_t f) { return perm(f << 8, f, 0x090B080Au); }
// 0xFF in every byte whose PAIR PARTNER (byte ^ 1) has bit 7 set in f
SPARQ_HD uint32_t expand_bit7_swapped(uint32_t f) { return perm(f << 8, f, 0x0B090A08u); }
// bit 7 of each byte = (byte != 0); other bits unspecified
SPARQ_HD uint32_t nonzero_flag(uint32_t v) { return lerp(v, 0xFFFFFFFFu, 0u); }

SPARQ_HD uint32_t low_mask(uint32_t selA, uint32_t selB, uint32_t a_hi, uint32_t a_lo, uint32_t b_hi,
                           uint32_t b_lo) {
    return perm(a_hi, a_lo, selA) | perm(b_hi, b_lo, selB);
}

// Trim four packed activations.  ROUND: "+R".  PAIR: vSPARQ on.  WIDE: a zero
// partner grants a 2n-bit window with 2n < 8 (n = 2, 3); with n = 4 the value
// simply stays as it is.
template <bool ROUND, bool PAIR, bool WIDE>
SPARQ_HD uint32_t trim4(uint32_t x, const TrimLuts& L) {
    const uint32_t selA = (x >> 5) & 0x07070707u;
    const uint32_t selB = (x >> 2) & 0x07070707u;
    const uint32_t low_n = low_mask(selA, selB, L.a_hi, L.a_lo, L.b_hi, L.b_lo);
    uint32_t low = low_n;
    uint32_t wtop = 0;          // all bits up to the window top, per byte (only needed for ROUND)
    if (PAIR) {
        // pm: bytes whose partner is non-zero (they are trimmed to n bits)
        const uint32_t pm = expand_bit7_swapped(nonzero_flag(x));
        if (WIDE) {
            const uint32_t low_w = low_mask(selA, selB, L.wa_hi, L.wa_lo, L.wb_hi, L.wb_lo);
            low = bfi(pm, low_n, low_w);
            if (ROUND) wtop = bfi(pm, (low_n << L.n) | L.ones_n, (low_w << L.n2) | L.ones_w);
        } else {
            low = low_n & pm;
            if (ROUND) wtop = (low << L.n) | L.ones_n;
        }
    } else if (ROUND) {
        wtop = (low << L.n) | L.ones_n;
    }
    const uint32_t fl = x & ~low;
    if (!ROUND) return fl;
    const uint32_t below_half = low & (low >> 1);      // residual bits under the rounding bit
    const uint32_t half = low ^ below_half;            // 2^(s-1), or 0 when s == 0
    const uint32_t zeros = ~x & (wtop ^ below_half);   // zero bits of x among window + rounding bit
    const uint32_t may_round = expand_bit7(nonzero_flag(zeros));   // 0 => window full and rounding bit set
    const uint32_t r = x & half & may_round;
    return fl + (r << 1);
}

// n = 4 with rounding: the saturation test is a byte-wise compare against a per-region
// threshold (one table lookup + v_lerp_u8), and rounding is "add the half bit, then drop the
// residual": x + 2^(s-1) cannot leave the byte unless the value saturates.
template <bool PAIR>
SPARQ_HD uint32_t trim4_round_n4(uint32_t x, const TrimLuts& L) {
    const uint32_t selA = (x >> 5) & 0x07070707u;
    const uint32_t selB = (x >> 2) & 0x07070707u;
    uint32_t low = low_mask(selA, selB, L.a_hi, L.a_lo, L.b_hi, L.b_lo);
    if (PAIR) low &= expand_bit7_swapped(nonzero_flag(x));
    const uint32_t half = low & ~(low >> 1);
    const uint32_t sat = expand_bit7(lerp(x, perm(L.ncap_hi, L.ncap_lo, selA), 0u));   // x + (256 - cap) >= 256
    return (x + (half & ~sat)) & ~low;
}

// Runtime-dispatched form for code that is not performance critical.
SPARQ_HD uint32_t trim4_any(uint32_t x, const TrimLuts& L, bool round_nearest, bool pair) {
    if (L.n >= 8) return x;
    const bool wide = pair && L.n < 4;
    if (round_nearest && L.n == 4) return pair ? trim4_round_n4<true>(x, L) : trim4_round_n4<false>(x, L);
    if (round_nearest) {
        if (!pair) return trim4<true, false, false>(x, L);
        return wide ? trim4<true, true, true>(x, L) : trim4<true, true, false>(x, L);
    }
    if (!pair) return trim4<false, false, false>(x, L);
    return wide ? trim4<false, true, true>(x, L) : trim4<false, true, false>(x, L);
}

}  // namespace sparq
