// Host-side helpers shared by the translation units of libsparq: argument
// validation, the packed-weight layout and launch bookkeeping.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/sparq.h"
#include "sparq_swar.h"

namespace sparq {

constexpr int kChunk = 16;        // bytes one lane feeds to an int8 matrix instruction
constexpr int kStepK = 64;        // reduction bytes per main-loop step
constexpr int kPadN = 256;        // packed output channels are padded to this

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

// ---- mode -----------------------------------------------------------------
// A set of placements for w-bit windows is usable when the lookup tables of sparq_swar.h can be built from it:
// every leading-one position 0..7 finds a placement, position 0 gets shift 0 (values below 2^w pass unchanged),
// and no placement pushes a window past bit 7.
inline bool placements_cover_a_byte(int w, uint32_t S) {
    if (S & ~((2u << (8 - w)) - 1u)) return false;
    if (trim_shift_for(0, w, S) != 0) return false;
    for (int p = 1; p < 8; ++p)
        if (trim_shift_for(p, w, S) > 8 - w) return false;
    return true;
}

inline bool mode_valid(const sparq_mode* m) {
    if (!m) return false;
    if (m->window_bits == 8) return true;
    if (m->window_bits < 2 || m->window_bits > 4) return false;
    if ((unsigned)m->round_nearest > 1u || (unsigned)m->pair > 1u) return false;
    if (!placements_cover_a_byte(m->window_bits, m->shift_mask)) return false;
    // vSPARQ: a value whose partner is zero gets a window of twice the width (the whole byte for 4-bit windows)
    return !m->pair || placements_cover_a_byte(2 * m->window_bits, wide_shift_mask(m->window_bits, m->shift_mask));
}

// Which compiled variant of the trim a mode needs.
enum TrimKind : int {
    kTrimNone = 0,
    kTrimFloor, kTrimFloorPair, kTrimFloorPairWide,
    kTrimRound, kTrimRoundPairWide,        // 2- and 3-bit windows
    kTrimRound4, kTrimRoundPair4,          // 4-bit windows: cheaper saturation test
    kTrimKinds
};

inline TrimKind trim_kind(const sparq_mode* m) {
    if (m->window_bits == 8) return kTrimNone;
    const bool wide = m->pair && m->window_bits < 4;
    if (m->round_nearest && m->window_bits == 4) return m->pair ? kTrimRoundPair4 : kTrimRound4;
    if (m->round_nearest) return wide ? kTrimRoundPairWide : kTrimRound;
    return !m->pair ? kTrimFloor : (wide ? kTrimFloorPairWide : kTrimFloorPair);
}

template <int KIND>
__device__ __forceinline__ uint32_t trim4_kind(uint32_t x, const TrimLuts& L) {
    if constexpr (KIND == kTrimNone) return x;
    else if constexpr (KIND == kTrimFloor) return trim4<false, false, false>(x, L);
    else if constexpr (KIND == kTrimFloorPair) return trim4<false, true, false>(x, L);
    else if constexpr (KIND == kTrimFloorPairWide) return trim4<false, true, true>(x, L);
    else if constexpr (KIND == kTrimRound) return trim4<true, false, false>(x, L);
    else if constexpr (KIND == kTrimRound4) return trim4_round_n4<false>(x, L);
    else if constexpr (KIND == kTrimRoundPair4) return trim4_round_n4<true>(x, L);
    else return trim4<true, true, true>(x, L);
}

// ---- convolution geometry and packed weights --------------------------------
struct ConvGeom {
    int B, H, W, C, N, KH, KW, sh, sw, ph, pw;
    int Ho, Wo;
    int64_t M;
    int Cp;          // channels padded to a multiple of 16 (what the kernel loads)
    int Cq;          // one filter tap's extent in the packed weights: C padded to 64 (to 16 when C <= 32)
    int K;           // KH*KW*C   (the method's dot-product length)
    int Kk;          // KH*KW*Cq  (what the kernel contracts over; with C > 32 every 64-byte step lies inside one tap)
    int Kp;          // Kk padded to kStepK
    int Np;          // N padded to kPadN
    size_t w_off;    // byte offset of the weight tiles inside the packed buffer
    size_t packed_bytes;
    size_t x_bytes;
    // Pixel folding for layers with at most 4 channels (a network's first convolution): four
    // neighbouring pixels of a row, each padded to 4 channels, become one 16-channel "super-pixel".
    // Output columns split into fold_p = 4 / stride_w classes by their position inside a super-pixel;
    // class p of output channel n becomes output channel p*N + n of a stride-1 convolution over
    // super-pixels with fold_kw taps per row -- and [M/fold_p][fold_p*N] is the same memory as [M][N].
    bool fold;
    int fold_p, fold_kw, fold_kw_min, fold_pw;
};

inline int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }


inline bool conv_geom(const sparq_conv_desc* d, ConvGeom* g) {
    if (!d) return false;
    if (d->B <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->N <= 0 || d->KH <= 0 || d->KW <= 0 ||
        d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0)
        return false;
    if ((int64_t)d->H + 2 * (int64_t)d->pad_h < d->KH || (int64_t)d->W + 2 * (int64_t)d->pad_w < d->KW) return false;
    g->B = d->B; g->H = d->H; g->W = d->W; g->C = d->C; g->N = d->N; g->KH = d->KH; g->KW = d->KW;
    g->sh = d->stride_h; g->sw = d->stride_w; g->ph = d->pad_h; g->pw = d->pad_w;
    g->Ho = (d->H + 2 * d->pad_h - d->KH) / d->stride_h + 1;
    g->Wo = (d->W + 2 * d->pad_w - d->KW) / d->stride_w + 1;
    g->M = (int64_t)d->B * g->Ho * g->Wo;
    const int64_t K = (int64_t)d->KH * d->KW * d->C;
    // 255 * 127 * K must stay inside int32 (it also bounds the offset form 128 * 127 * K)
    if (K * 255 * 127 > 2147483647LL) return false;
    g->K = (int)K;
    g->Cp = (int)round_up(d->C, kChunk);
    g->Cq = d->C > 32 ? (int)round_up(d->C, kStepK) : g->Cp;     // few channels: taps stay densely packed
    const int64_t Kk = (int64_t)d->KH * d->KW * g->Cq;
    if (Kk > (1 << 24)) return false;
    g->Kk = (int)Kk;
    g->Kp = (int)round_up(Kk, kStepK);
    g->Np = (int)round_up(d->N, kPadN);
    g->w_off = (size_t)round_up((int64_t)g->Np * 4, 256);
    g->packed_bytes = g->w_off + (size_t)g->Kp * (size_t)g->Np;
    g->x_bytes = (size_t)d->B * d->H * d->W * (size_t)d->C;
    g->fold = false;
    g->fold_p = 1; g->fold_kw = d->KW; g->fold_kw_min = 0; g->fold_pw = d->pad_w;
    if (d->C <= 4 && d->W % 4 == 0 && 4 % d->stride_w == 0 && d->KH * d->KW > 1) {
        const int P = 4 / d->stride_w;
        const int kw_min = floor_div(-d->pad_w, 4);
        const int kw_max = floor_div(d->stride_w * (P - 1) - d->pad_w + d->KW - 1, 4);
        const int KWf = kw_max - kw_min + 1, pwf = -kw_min;
        if (g->Wo % P == 0 && d->W / 4 + 2 * pwf - KWf + 1 == g->Wo / P) {
            g->fold = true;
            g->fold_p = P; g->fold_kw = KWf; g->fold_kw_min = kw_min; g->fold_pw = pwf;
            // sizes of the packed weights of the folded problem: 16 channels per tap, fold_p * N outputs
            const int64_t Kf = (int64_t)d->KH * KWf * 16;
            g->Kp = (int)round_up(Kf, kStepK);
            g->Np = (int)round_up((int64_t)P * d->N, kPadN);
            g->w_off = (size_t)round_up((int64_t)g->Np * 4, 256);
            g->packed_bytes = g->w_off + (size_t)g->Kp * (size_t)g->Np;
        }
    }
    return true;
}

// The convolution the kernels see when `g` is folded: super-pixels of 16 channels, stride 1 along W.
inline ConvGeom folded_view(const ConvGeom& g) {
    ConvGeom f = g;
    f.W = g.W / 4; f.C = 16; f.Cp = 16; f.Cq = 16;
    f.N = g.fold_p * g.N;
    f.KW = g.fold_kw; f.sw = 1; f.pw = g.fold_pw;
    f.Wo = g.Wo / g.fold_p;
    f.M = g.M / g.fold_p;
    f.Kk = g.KH * g.fold_kw * 16;
    f.x_bytes = (size_t)g.B * g.H * g.W * 4;
    f.fold = false;
    return f;
}

#if defined(__HIPCC__)
// Requantised result (the arithmetic the byte output is defined by): fp32 product, round to nearest even, clamp.
__device__ __forceinline__ uint32_t requant_u8(int32_t r, float factor) {
    const float f = __builtin_rintf(__fmul_rn((float)r, factor));
    return (uint32_t)__builtin_fminf(__builtin_fmaxf(f, 0.0f), 255.0f);
}

// 4 x 4 byte transpose inside every group of four neighbouring lanes.  Lane t of a group holds word P_t
// (byte k = its value for row k); afterwards lane t holds byte t of P_0, P_1, P_2, P_3 (the four lanes'
// values for row t).  The matrix instruction leaves a lane with four consecutive rows of one channel; after
// the transpose it has four consecutive channels of one row, i.e. one 32-bit store instead of four byte
// stores.  sel_a / sel_d depend on the lane only (quad_transpose_selectors).
// Four requantised results packed into one word (byte k from r[k]): the conversion instruction rounds to
// nearest even and saturates to [0, 255] by itself.
__device__ __forceinline__ uint32_t requant_u8x4(int32_t r0, int32_t r1, int32_t r2, int32_t r3, float factor) {
    uint32_t w = __builtin_amdgcn_cvt_pk_u8_f32(__fmul_rn((float)r0, factor), 0, 0);
    w = __builtin_amdgcn_cvt_pk_u8_f32(__fmul_rn((float)r1, factor), 1, w);
    w = __builtin_amdgcn_cvt_pk_u8_f32(__fmul_rn((float)r2, factor), 2, w);
    return __builtin_amdgcn_cvt_pk_u8_f32(__fmul_rn((float)r3, factor), 3, w);
}

// Cache policy of the int32 / fp32 result stores of the convolution kernels: non-temporal.  These results are four
// bytes per output, written once and not read again by the int8 path (the next layer reads the requantised bytes,
// which keep the ordinary policy); layers bound by this stream run 6-15 % faster, the others do not change.
constexpr int kResultStorePolicy = 2;            // the `nt` bit of the buffer-store cache policy

struct QuadSel { uint32_t a, d; };
__device__ __forceinline__ QuadSel quad_transpose_selectors(int lane) {
    const uint32_t t = (uint32_t)lane & 3u;
    QuadSel q;
    q.a = t | ((4u + t) << 8);                    // byte t of the low word, byte t of the high word
    static constexpr uint32_t code[4] = {0u, 1u, 4u, 5u};   // own, lane^1 (low pair); lane^2, lane^3 (high pair)
    q.d = 0;
#pragma unroll
    for (uint32_t s = 0; s < 4; ++s) q.d |= code[s ^ t] << (8 * s);
    return q;
}
__device__ __forceinline__ uint32_t quad_transpose_bytes(uint32_t own, QuadSel sel) {
    const uint32_t a = (uint32_t)__builtin_amdgcn_mov_dpp((int)own, 0xB1, 0xF, 0xF, true);   // from lane ^ 1
    const uint32_t b = (uint32_t)__builtin_amdgcn_mov_dpp((int)own, 0x4E, 0xF, 0xF, true);   // from lane ^ 2
    const uint32_t c = (uint32_t)__builtin_amdgcn_mov_dpp((int)own, 0x1B, 0xF, 0xF, true);   // from lane ^ 3
    const uint32_t x = __builtin_amdgcn_perm(a, own, sel.a);     // [own.t, a.t, -, -]
    const uint32_t y = __builtin_amdgcn_perm(c, b, sel.a);       // [b.t, c.t, -, -]
    return __builtin_amdgcn_perm(y, x, sel.d);
}
#endif

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline sparq_status launch_status() { return hipGetLastError() == hipSuccess ? SPARQ_OK : SPARQ_ELAUNCH; }

// Per-device bookkeeping (kernel attributes set, CU counts) is kept in small tables indexed by the HIP device
// ordinal; ordinals past the table share its last slot, which only costs repeated attribute calls.
constexpr int kMaxDevices = 16;
inline int current_device_slot() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) dev = 0;
    return dev < kMaxDevices ? dev : kMaxDevices - 1;
}

// Number of compute units of the current device (queried once per device; concurrent first calls both query).
inline int device_cu_count() {
    static std::atomic<int> cus[kMaxDevices];
    const int slot = current_device_slot();
    int n = cus[slot].load(std::memory_order_relaxed);
    if (n == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 256;
        n = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        cus[slot].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Implemented in sparq_elementwise.hip: trimmed copy of x with channels padded to Cp.
sparq_status launch_trim_pad(const uint8_t* x, uint8_t* xp, int64_t pixels, int C, int Cp,
                             const sparq_mode* mode, hipStream_t stream);


// Implemented in sparq_sparse24.hip: the expanded activation tensor (16 bytes per group of four channels) and the
// dense (expand: 16 bytes per group, else 4) form of 2:4 compressed weights.
sparq_status launch_sparse24_expand_act(const uint8_t* x, uint8_t* xe, int64_t pixels, int C, const sparq_mode* mode,
                                        hipStream_t stream);
sparq_status launch_sparse24_expand_weights(const int8_t* vals, const uint8_t* idx, int8_t* dense, int64_t groups, bool expand,
                                            hipStream_t stream);
// ... and the operands of the sparse matrix instruction (16 kept bytes + one word of positions per 32 reduction
// indices) from dense weights [N][taps][C] with at most two non-zeros per aligned group of four channels.
sparq_status launch_sparse24_pack_operand(const int8_t* dense, uint8_t* vals, uint32_t* pos, int N, int Np, int taps, int C,
                                          int Cq, hipStream_t stream);

// Implemented in sparq_packed_act.hip: the 8-bit values a packed activation tensor encodes.
sparq_status launch_unpack_act(const void* packed, uint8_t* y, int64_t rows, int C, const sparq_mode* mode, int group,
                               hipStream_t stream);


}  // namespace sparq
