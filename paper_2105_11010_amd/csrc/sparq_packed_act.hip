// Packed storage of trimmed activations: what SPARQ's multiplier consumes (Eq. 4) instead of 8-bit values.
//
// Section 3.1: an n-bit window travels with an identifier of its position; Section 5.1: per n-bit datum a
// ShiftCtrl field and, with vSPARQ, a 1-bit MuxCtrl that names the weight the datum multiplies; Section 6:
// ShiftCtrl may be shared by a number of activations.  A pair of channels (2j, 2j+1) is stored as two data:
//   both values non-zero (or vSPARQ off): their two windows, each steered to its own channel;
//   second value zero, else first value zero (the case order of Eq. 2): the other value's 2n-bit window as a
//   high half (shift t+n) and a low half (shift t), both steered to that value's channel.
// A channel's value is the sum of datum << shift over the data steered to it.
//
// Record layout (32 channels of one row, the last record of a row zero-filled; little-endian 32-bit words):
//   data      n words          datum k in bits [k*n, k*n+n)
//   ShiftCtrl ceil(F*sb/32) w. field f in bits [f*sb, f*sb+sb): rank of the shift among the allowed ones;
//                              sb = bits to number them; F = 32 / group fields (group = 1: one per datum)
//   MuxCtrl   1 word           bit k: datum k goes to the odd channel of its pair (absent with vSPARQ off)
// group > 1 (vSPARQ off only): one shift per group of consecutive channels, the placement bSPARQ picks for the
// group's largest value; every value of the group is trimmed at that shift (floor, or round half up saturating).
//
// One lane handles one record.  The window fields are recomputed from the TRIMMED byte: its leading one still
// lies in the window the untrimmed value selected (rounding saturates inside the window), so shift and datum
// follow from two 8-entry tables indexed by the leading-one position.
#include "sparq_common.h"

namespace sparq {

namespace {

constexpr int kRecChannels = 32;
constexpr int kPkThreads = 256;

struct PackLuts {            // 4 bits per entry, entry p = leading-one position 0..7 (or ShiftCtrl code for the last)
    uint32_t shift_n, code_n;            // n-bit window: its shift, the ShiftCtrl code of that shift
    uint32_t shift_w, code_hi, code_lo;  // 2n-bit window of a value whose partner is zero: shift t, codes of t+n and t
    uint32_t shift_of_code;              // decoder: shift of ShiftCtrl code c
    TrimLuts trim;
    int round_nearest, pair;
};

int popcount_below(uint32_t S, int t) { return __builtin_popcount(S & ((1u << t) - 1u)); }

int shift_ctrl_bits(uint32_t S) {
    int bits = 0;
    while ((1 << bits) < __builtin_popcount(S)) ++bits;
    return bits;
}

PackLuts make_pack_luts(const sparq_mode* m) {
    PackLuts L{};
    const int n = m->window_bits;
    const uint32_t S = m->shift_mask, W = wide_shift_mask(n, S);
    for (int p = 0; p < 8; ++p) {
        const int s = trim_shift_for(p, n, S);
        L.shift_n |= (uint32_t)(s & 15) << (4 * p);
        L.code_n |= (uint32_t)popcount_below(S, s) << (4 * p);
        if (m->pair) {
            const int t = trim_shift_for(p, 2 * n, W);
            L.shift_w |= (uint32_t)(t & 15) << (4 * p);
            L.code_hi |= (uint32_t)popcount_below(S, t + n) << (4 * p);
            L.code_lo |= (uint32_t)popcount_below(S, t) << (4 * p);
        }
    }
    int code = 0;
    for (int t = 0; t < 8; ++t)
        if ((S >> t) & 1u) L.shift_of_code |= (uint32_t)t << (4 * code++);
    L.trim = make_luts(n, S);
    L.round_nearest = m->round_nearest;
    L.pair = m->pair;
    return L;
}

__device__ __forceinline__ uint32_t nib(uint32_t table, uint32_t index) { return (table >> (4 * index)) & 15u; }
__device__ __forceinline__ uint32_t top_bit(uint32_t v) { return v ? 31u - (uint32_t)__builtin_clz(v) : 0u; }

// OR `value` (nbits wide) into a little-endian bit string of WORDS words at a position known at compile time.
template <int WORDS>
__device__ __forceinline__ void put_field(uint32_t (&area)[WORDS], int pos, int nbits, uint32_t value) {
    const int w = pos >> 5, off = pos & 31;
    area[w] |= value << off;
    if (off + nbits > 32 && w + 1 < WORDS) area[w + 1] |= value >> (32 - off);
}
template <int WORDS>
__device__ __forceinline__ uint32_t get_field(const uint32_t (&area)[WORDS], int pos, int nbits) {
    const int w = pos >> 5, off = pos & 31;
    uint32_t v = area[w] >> off;
    if (off + nbits > 32 && w + 1 < WORDS) v |= area[w + 1] << (32 - off);
    return v & ((1u << nbits) - 1u);
}
// The same at a position only known at run time (shared-shift fields): the word is picked by comparisons so that
// the array stays in registers.
template <int WORDS>
__device__ __forceinline__ void put_field_rt(uint32_t (&area)[WORDS], int pos, int nbits, uint32_t value) {
    const int w = pos >> 5, off = pos & 31;
    const uint32_t lo = value << off, hi = (off + nbits > 32) ? value >> (32 - off) : 0u;
#pragma unroll
    for (int i = 0; i < WORDS; ++i) area[i] |= (w == i ? lo : 0u) | (w + 1 == i ? hi : 0u);
}
template <int WORDS>
__device__ __forceinline__ uint32_t get_field_rt(const uint32_t (&area)[WORDS], int pos, int nbits) {
    const int w = pos >> 5, off = pos & 31;
    uint32_t a = 0, b = 0;
#pragma unroll
    for (int i = 0; i < WORDS; ++i) {
        a = (w == i) ? area[i] : a;
        b = (w + 1 == i) ? area[i] : b;
    }
    const uint32_t v = (a >> off) | ((off + nbits > 32) ? b << (32 - off) : 0u);
    return v & ((1u << nbits) - 1u);
}

// 32 channels of row r starting at channel c0 as eight words (channels past C read as zero).
__device__ __forceinline__ void load_record_bytes(const uint8_t* x, int64_t r, int C, int c0, bool fast, uint32_t (&w)[8]) {
    const uint8_t* src = x + r * C + c0;
    if (fast) {
        const uint4 a = reinterpret_cast<const uint4*>(src)[0], b = reinterpret_cast<const uint4*>(src)[1];
        w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t v = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (c0 + 4 * i + j < C) v |= (uint32_t)src[4 * i + j] << (8 * j);
            w[i] = v;
        }
    }
}

// N window bits, SB ShiftCtrl bits.  group == 1: per-value fields (and MuxCtrl when L.pair); group > 1: shared shift.
template <int N, int SB>
__global__ __launch_bounds__(kPkThreads) void pack_act_kernel(const uint8_t* __restrict__ x, uint32_t* __restrict__ packed,
                                                               int64_t rows, int C, int nrec, int group, int rec_words,
                                                               bool fast, PackLuts L) {
    const int64_t total = rows * nrec;
    const int64_t stride = (int64_t)gridDim.x * kPkThreads;
    const uint32_t qmask = (1u << N) - 1u;
    for (int64_t idx = (int64_t)blockIdx.x * kPkThreads + threadIdx.x; idx < total; idx += stride) {
        const int64_t r = idx / nrec;
        const int c0 = (int)(idx - r * nrec) * kRecChannels;
        uint32_t w[8];
        load_record_bytes(x, r, C, c0, fast, w);
        uint32_t data[N] = {}, shifts[SB] = {}, mux = 0;
        if (group == 1) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t t4 = trim4_any(w[i], L.trim, L.round_nearest != 0, L.pair != 0);
#pragma unroll
                for (int h = 0; h < 2; ++h) {                       // the two pairs of the word
                    const int k = 4 * i + 2 * h;                    // datum index of the pair's first channel
                    const uint32_t ta = (t4 >> (16 * h)) & 255u, tb = (t4 >> (16 * h + 8)) & 255u;
                    uint32_t d0, d1, c0_, c1_, m0 = 0, m1 = 1;
                    if (L.pair && (ta == 0 || tb == 0)) {
                        const uint32_t owner = tb == 0 ? 0u : 1u, v = owner ? tb : ta, p = top_bit(v);
                        const uint32_t t = nib(L.shift_w, p);
                        d0 = (v >> (t + N)) & qmask;
                        d1 = (v >> t) & qmask;
                        c0_ = nib(L.code_hi, p);
                        c1_ = nib(L.code_lo, p);
                        m0 = m1 = owner;
                    } else {
                        const uint32_t pa = top_bit(ta), pb = top_bit(tb);
                        d0 = ta >> nib(L.shift_n, pa);
                        d1 = tb >> nib(L.shift_n, pb);
                        c0_ = nib(L.code_n, pa);
                        c1_ = nib(L.code_n, pb);
                    }
                    put_field(data, k * N, N, d0);
                    put_field(data, (k + 1) * N, N, d1);
                    put_field(shifts, k * SB, SB, c0_);
                    put_field(shifts, (k + 1) * SB, SB, c1_);
                    mux |= (m0 << k) | (m1 << (k + 1));
                }
            }
        } else {
            // shared shift: the group's largest value picks the placement, every value is trimmed there.
            // Group maxima at every power-of-two size (2, 4, 8, 16, 32 channels); the run-time size picks one.
            uint32_t m1[16], m2[8], m3[4], m4[2], m5;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t b0 = w[i] & 255u, b1 = (w[i] >> 8) & 255u, b2 = (w[i] >> 16) & 255u, b3 = w[i] >> 24;
                m1[2 * i] = b0 > b1 ? b0 : b1;
                m1[2 * i + 1] = b2 > b3 ? b2 : b3;
                m2[i] = m1[2 * i] > m1[2 * i + 1] ? m1[2 * i] : m1[2 * i + 1];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) m3[i] = m2[2 * i] > m2[2 * i + 1] ? m2[2 * i] : m2[2 * i + 1];
            m4[0] = m3[0] > m3[1] ? m3[0] : m3[1];
            m4[1] = m3[2] > m3[3] ? m3[2] : m3[3];
            m5 = m4[0] > m4[1] ? m4[0] : m4[1];
#pragma unroll
            for (int j = 0; j < 16; ++j) {                              // pairs of channels: a group never splits one
                const uint32_t top = group == 2 ? m1[j] : group == 4 ? m2[j >> 1] : group == 8 ? m3[j >> 2]
                                   : group == 16 ? m4[j >> 3] : m5;
                const uint32_t p = top_bit(top), s_ = nib(L.shift_n, p);
                if (((2 * j) & (group - 1)) == 0) put_field_rt(shifts, (2 * j / group) * SB, SB, nib(L.code_n, p));
                const uint32_t half = (L.round_nearest && s_ > 0) ? 1u << (s_ - 1) : 0u;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int k = 2 * j + e;
                    const uint32_t v = (w[k >> 2] >> (8 * (k & 3))) & 255u;
                    uint32_t q = (v + half) >> s_;
                    q = q > qmask ? qmask : q;
                    put_field(data, k * N, N, q);
                }
            }
        }
        uint32_t* dst = packed + idx * rec_words;
        int o = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) dst[o++] = data[i];
        const int sw = rec_words - N - (L.pair ? 1 : 0);
#pragma unroll
        for (int i = 0; i < SB; ++i)
            if (i < sw) dst[o++] = shifts[i];
        if (L.pair) dst[o] = mux;
    }
}

template <int N, int SB>
__global__ __launch_bounds__(kPkThreads) void unpack_act_kernel(const uint32_t* __restrict__ packed, uint8_t* __restrict__ y,
                                                                 int64_t rows, int C, int nrec, int group, int rec_words,
                                                                 bool fast, PackLuts L) {
    const int64_t total = rows * nrec;
    const int64_t stride = (int64_t)gridDim.x * kPkThreads;
    for (int64_t idx = (int64_t)blockIdx.x * kPkThreads + threadIdx.x; idx < total; idx += stride) {
        const int64_t r = idx / nrec;
        const int c0 = (int)(idx - r * nrec) * kRecChannels;
        const uint32_t* src = packed + idx * rec_words;
        uint32_t data[N], shifts[SB] = {}, mux = 0;
        int o = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) data[i] = src[o++];
        const int sw = rec_words - N - (L.pair ? 1 : 0);
#pragma unroll
        for (int i = 0; i < SB; ++i)
            if (i < sw) shifts[i] = src[o++];
        if (L.pair) mux = src[o];
        uint32_t w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t word = 0;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int k = 4 * i + 2 * h;
                uint32_t v[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const uint32_t q = get_field(data, (k + e) * N, N);
                    const uint32_t code = group == 1 ? get_field(shifts, (k + e) * SB, SB)
                                                     : get_field_rt(shifts, ((k + e) / group) * SB, SB);
                    v[e] = q << nib(L.shift_of_code, code);
                }
                // Eq. 4: each datum adds to the channel its MuxCtrl names (own channel when vSPARQ is off)
                const uint32_t m0 = L.pair ? (mux >> k) & 1u : 0u, m1 = L.pair ? (mux >> (k + 1)) & 1u : 1u;
                const uint32_t even = (m0 ? 0u : v[0]) + (m1 ? 0u : v[1]);
                const uint32_t odd = (m0 ? v[0] : 0u) + (m1 ? v[1] : 0u);
                word |= ((even & 255u) | ((odd & 255u) << 8)) << (16 * h);
            }
            w[i] = word;
        }
        uint8_t* dst = y + r * C + c0;
        if (fast) {
            reinterpret_cast<uint4*>(dst)[0] = make_uint4(w[0], w[1], w[2], w[3]);
            reinterpret_cast<uint4*>(dst)[1] = make_uint4(w[4], w[5], w[6], w[7]);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (c0 + 4 * i + j < C) dst[4 * i + j] = (uint8_t)(w[i] >> (8 * j));
        }
    }
}

int grid_for(int64_t items) {
    int64_t blocks = (items + kPkThreads - 1) / kPkThreads;
    if (blocks > 256 * 16) blocks = 256 * 16;
    return (int)(blocks < 1 ? 1 : blocks);
}

// Record size in 32-bit words; 0: this mode / group has no packed form.
int record_words(const sparq_mode* mode, int group) {
    if (!mode_valid(mode) || mode->window_bits == 8) return 0;
    if (group < 1 || group > kRecChannels || kRecChannels % group != 0 || (group > 1 && mode->pair)) return 0;
    const int sb = shift_ctrl_bits(mode->shift_mask);
    return mode->window_bits + (kRecChannels / group * sb + 31) / 32 + (mode->pair ? 1 : 0);
}

template <bool PACK>
sparq_status launch_codec(const void* in, void* out, int64_t rows, int C, const sparq_mode* mode, int group, hipStream_t s) {
    const int words = record_words(mode, group);
    const int nrec = (C + kRecChannels - 1) / kRecChannels;
    if (rows == 0) return SPARQ_OK;
    const PackLuts L = make_pack_luts(mode);
    const int n = mode->window_bits, sb = shift_ctrl_bits(mode->shift_mask);
    const void* bytes = PACK ? in : out;
    const bool fast = C % kRecChannels == 0 && aligned(bytes, 16);
    const int grid = grid_for(rows * nrec);
#define SPARQ_CODEC_CASE(NN, SS)                                                                                             \
    if (n == NN && sb == SS) {                                                                                               \
        if (PACK)                                                                                                            \
            pack_act_kernel<NN, SS><<<grid, kPkThreads, 0, s>>>(static_cast<const uint8_t*>(in), static_cast<uint32_t*>(out), \
                                                                rows, C, nrec, group, words, fast, L);                       \
        else                                                                                                                 \
            unpack_act_kernel<NN, SS><<<grid, kPkThreads, 0, s>>>(static_cast<const uint32_t*>(in), static_cast<uint8_t*>(out), \
                                                                  rows, C, nrec, group, words, fast, L);                     \
        return launch_status();                                                                                              \
    }
    SPARQ_CODEC_CASE(4, 3) SPARQ_CODEC_CASE(4, 2) SPARQ_CODEC_CASE(4, 1)
    SPARQ_CODEC_CASE(3, 3) SPARQ_CODEC_CASE(3, 2) SPARQ_CODEC_CASE(3, 1)
    SPARQ_CODEC_CASE(2, 3) SPARQ_CODEC_CASE(2, 2) SPARQ_CODEC_CASE(2, 1)
#undef SPARQ_CODEC_CASE
    return SPARQ_EUNSUPPORTED;
}

}  // namespace

sparq_status launch_unpack_act(const void* packed, uint8_t* y, int64_t rows, int C, const sparq_mode* mode, int group,
                               hipStream_t s) {
    return launch_codec<false>(packed, y, rows, C, mode, group, s);
}

}  // namespace sparq

using namespace sparq;

extern "C" size_t sparq_packed_act_bytes(int64_t rows, int32_t C, const sparq_mode* mode, int32_t group) {
    const int words = record_words(mode, group);
    if (words == 0 || rows < 0 || C <= 0) return 0;
    return (size_t)rows * (size_t)((C + kRecChannels - 1) / kRecChannels) * (size_t)words * 4;
}

extern "C" sparq_status sparq_pack_act(const uint8_t* x, void* packed, size_t packed_bytes, int64_t rows, int32_t C,
                                       const sparq_mode* mode, int32_t group, void* stream) {
    if (rows < 0 || C <= 0 || record_words(mode, group) == 0) return SPARQ_EINVAL;
    if (rows == 0) return SPARQ_OK;                      // nothing to do (the pointers are not looked at)
    if (!x || !packed || !aligned(packed, 4)) return SPARQ_EINVAL;
    if (packed_bytes < sparq_packed_act_bytes(rows, C, mode, group)) return SPARQ_EWORKSPACE;
    return launch_codec<true>(x, packed, rows, C, mode, group, static_cast<hipStream_t>(stream));
}

extern "C" sparq_status sparq_unpack_act(const void* packed, size_t packed_bytes, uint8_t* y, int64_t rows, int32_t C,
                                         const sparq_mode* mode, int32_t group, void* stream) {
    if (rows < 0 || C <= 0 || record_words(mode, group) == 0) return SPARQ_EINVAL;
    if (rows == 0) return SPARQ_OK;
    if (!packed || !y || !aligned(packed, 4)) return SPARQ_EINVAL;
    if (packed_bytes < sparq_packed_act_bytes(rows, C, mode, group)) return SPARQ_EWORKSPACE;
    return launch_codec<false>(packed, y, rows, C, mode, group, static_cast<hipStream_t>(stream));
}
