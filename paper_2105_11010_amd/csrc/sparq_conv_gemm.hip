// Fused SPARQ convolution-as-GEMM for gfx950.
//
//   acc[m][n] = sum_k T(x)[m, k] * w[n][k]          (Eq. 1 over trimmed activations)
//
// The im2col matrix is never materialised: every workgroup gathers its
// activation tile straight from the NHWC tensor with 128-bit loads (one load =
// 16 consecutive channels of one pixel = 8 vSPARQ pairs inside one lane), trims
// the four packed words in registers (sparq_swar.h), flips them to signed
// (x - 128, a single xor) and stages them in LDS.  Weights arrive pre-packed in
// exactly the order the LDS tile wants.  The contraction runs on
// v_mfma_i32_32x32x32_i8; the epilogue adds back 128 * sum_k w[n][k], which
// makes the result exact in int32, and optionally applies the per-channel
// dequantisation factor (Section 5).
//
// Operand roles: the weights are the matrix instruction's row operand and the
// activations its column operand, so every lane ends up owning four
// consecutive output channels of one output pixel and the epilogue writes
// 128-bit words.
//
// This mirrors the paper's placement of the trimming unit in front of the
// array (Section 5: it runs at a much lower rate than the multipliers): an
// activation is trimmed once when its tile is loaded and then reused for all
// output channels the workgroup covers.
#include "sparq_common.h"

namespace sparq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

struct GemmParams {
    const uint8_t* x;        // activations, NHWC with C a multiple of 16
    const uint8_t* wpk;      // packed weight tiles
    const int32_t* colsum;   // sum_k w[n][k], Np entries
    int32_t* acc;            // [M][N] or null
    const float* scale;      // [N] or null
    float* out;              // [M][N] or null
    int64_t M;
    uint32_t x_bytes;
    int N, Np, Kk, nkb;
    int H, W, C, Ho, Wo, KH, KW, sh, sw, ph, pw;
    int tiles_m, tiles_n;
    TrimLuts luts;
};

constexpr uint32_t kInvalidOffset = 0x80000000u;   // beyond any buffer this kernel accepts (< 2 GiB)

template <int TM, int TN, int WGM, int WGN>
struct TileCfg {
    static constexpr int kTM = TM, kTN = TN, kWGM = WGM, kWGN = WGN;
    static constexpr int kThreads = 64 * WGM * WGN;
    static constexpr int kWTM = TM / WGM, kWTN = TN / WGN;      // per-wavefront tile
    static constexpr int kFM = kWTM / 32, kFN = kWTN / 32;      // 32x32 fragments per wavefront
    static constexpr int kAChunks = TM * 4 / kThreads;          // 16-byte loads per lane per step
    static constexpr int kBChunks = TN * 4 / kThreads;
    static constexpr int kLdsA = 4 * TM * kChunk;               // bytes per stage
    static constexpr int kLdsB = 4 * TN * kChunk;
    static constexpr int kLdsBytes = 2 * (kLdsA + kLdsB);
    static_assert(TM % (32 * WGM) == 0 && TN % (32 * WGN) == 0, "tile must split into 32x32 fragments");
    static_assert((TM * 4) % kThreads == 0 && (TN * 4) % kThreads == 0, "loads must divide evenly");
};

template <class Cfg, int KIND>
__global__ __launch_bounds__(Cfg::kThreads) void conv_gemm_kernel(const GemmParams p) {
    constexpr int TM = Cfg::kTM, TN = Cfg::kTN, NT = Cfg::kThreads;
    constexpr int FM = Cfg::kFM, FN = Cfg::kFN, AC = Cfg::kAChunks, BC = Cfg::kBChunks;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint8_t* const lds_a = lds;                       // [2][4][TM][16]
    uint8_t* const lds_b = lds + 2 * Cfg::kLdsA;      // [2][4][TN][16]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % Cfg::kWGM, wn = wave / Cfg::kWGM;

    // Workgroups are dealt round-robin to the 8 XCDs; renumber them so that each
    // XCD (one L2) works on a contiguous range of tiles, output-channel tiles of
    // the same activation rows next to each other.
    int bid = blockIdx.x;
    const int nblk = gridDim.x;
    if ((nblk & 7) == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int tile_n = bid % p.tiles_n;
    const int tile_m = bid / p.tiles_n;
    const int64_t m0 = (int64_t)tile_m * TM;
    const int n0 = tile_n * TN;

    // ---- activation gather bookkeeping (fixed per lane) ----
    const int kc = tid & 3;                  // which 16-byte chunk of the 64-byte step
    int32_t row_base[AC];                    // byte offset of (b, oy*sh-ph, ox*sw-pw, 0)
    int32_t row_iy[AC], row_ix[AC];
#pragma unroll
    for (int i = 0; i < AC; ++i) {
        int64_t m = m0 + (tid >> 2) + i * (NT / 4);
        if (m >= p.M) m = p.M - 1;
        const int ox = (int)(m % p.Wo);
        const int64_t t = m / p.Wo;
        const int oy = (int)(t % p.Ho);
        const int b = (int)(t / p.Ho);
        const int iy0 = oy * p.sh - p.ph, ix0 = ox * p.sw - p.pw;
        row_iy[i] = iy0;
        row_ix[i] = ix0;
        row_base[i] = (int32_t)((((int64_t)b * p.H + iy0) * p.W + ix0) * p.C);
    }
    // position of this lane's chunk inside the (kh, kw, c) reduction index
    int c0 = kc * kChunk, kw = 0, kh = 0;
    while (c0 >= p.C) { c0 -= p.C; if (++kw == p.KW) { kw = 0; ++kh; } }

    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.x), 0, (int)p.x_bytes, 0x00020000);

    v4u a_reg[AC];
    v4u b_reg[BC];

    auto load_tiles = [&](int kb) {
        const bool k_ok = kh < p.KH;                        // false only in the zero-padded K tail
        const int32_t tap_off = (kh * p.W + kw) * p.C + c0;
#pragma unroll
        for (int i = 0; i < AC; ++i) {
            const bool ok = k_ok && (unsigned)(row_iy[i] + kh) < (unsigned)p.H && (unsigned)(row_ix[i] + kw) < (unsigned)p.W;
            const uint32_t off = ok ? (uint32_t)(row_base[i] + tap_off) : kInvalidOffset;
            a_reg[i] = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, (int)off, 0, 0);   // out of range reads 0
        }
        const uint8_t* wsrc = p.wpk + (size_t)kb * 4 * p.Np * kChunk;
#pragma unroll
        for (int i = 0; i < BC; ++i) {
            const int q = i * NT + tid;
            const int bkc = q / TN, nn = q % TN;
            b_reg[i] = *reinterpret_cast<const v4u*>(wsrc + ((size_t)bkc * p.Np + n0 + nn) * kChunk);
        }
        // advance to the next 64-byte step
        c0 += kStepK;
        while (c0 >= p.C) { c0 -= p.C; if (++kw == p.KW) { kw = 0; ++kh; } }
    };

    auto store_tiles = [&](int stage) {
        uint8_t* sa = lds_a + stage * Cfg::kLdsA;
        uint8_t* sb = lds_b + stage * Cfg::kLdsB;
#pragma unroll
        for (int i = 0; i < AC; ++i) {
            v4u v = a_reg[i];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = trim4_kind<KIND>(v[j], p.luts) ^ 0x80808080u;
            const int row = (tid >> 2) + i * (NT / 4);
            *reinterpret_cast<v4u*>(sa + (kc * TM + row) * kChunk) = v;
        }
#pragma unroll
        for (int i = 0; i < BC; ++i) *reinterpret_cast<v4u*>(sb + (i * NT + tid) * kChunk) = b_reg[i];
    };

    v16i c[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) c[i][j][v] = 0;

    load_tiles(0);
    store_tiles(0);
    __syncthreads();

    const int l32 = lane & 31, lhi = lane >> 5;
    for (int kb = 0; kb < p.nkb; ++kb) {
        const int stage = kb & 1;
        const bool more = kb + 1 < p.nkb;
        if (more) load_tiles(kb + 1);
        const uint8_t* sa = lds_a + stage * Cfg::kLdsA;
        const uint8_t* sb = lds_b + stage * Cfg::kLdsB;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int fkc = ks * 2 + lhi;
            v4i wf[FN], af[FM];
#pragma unroll
            for (int j = 0; j < FN; ++j)
                wf[j] = *reinterpret_cast<const v4i*>(sb + (fkc * TN + wn * Cfg::kWTN + j * 32 + l32) * kChunk);
#pragma unroll
            for (int i = 0; i < FM; ++i)
                af[i] = *reinterpret_cast<const v4i*>(sa + (fkc * TM + wm * Cfg::kWTM + i * 32 + l32) * kChunk);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[j], af[i], c[i][j], 0, 0, 0);
        }
        if (more) store_tiles(stage ^ 1);
        __syncthreads();
    }

    // ---- epilogue: undo the -128 offset, store int32 and/or dequantised fp32 ----
    const bool vec_ok = (p.N & 3) == 0;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int64_t m = m0 + wm * Cfg::kWTM + i * 32 + l32;
        if (m >= p.M) continue;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * Cfg::kWTN + j * 32 + 8 * g + 4 * lhi;
                if (n >= p.N) continue;
                const v4i cs = *reinterpret_cast<const v4i*>(p.colsum + n);    // padded to Np, always readable
                v4i r;
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = c[i][j][4 * g + e] + 128 * cs[e];
                const int64_t o = m * p.N + n;
                if (vec_ok) {
                    if (p.acc) *reinterpret_cast<v4i*>(p.acc + o) = r;
                    if (p.out) {
                        const float4 s = *reinterpret_cast<const float4*>(p.scale + n);
                        float4 f;
                        f.x = __fmul_rn((float)r[0], s.x);
                        f.y = __fmul_rn((float)r[1], s.y);
                        f.z = __fmul_rn((float)r[2], s.z);
                        f.w = __fmul_rn((float)r[3], s.w);
                        *reinterpret_cast<float4*>(p.out + o) = f;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (n + e >= p.N) break;
                        if (p.acc) p.acc[o + e] = r[e];
                        if (p.out) p.out[o + e] = __fmul_rn((float)r[e], p.scale[n + e]);
                    }
                }
            }
        }
    }
}

template <class Cfg, int KIND>
static sparq_status launch_cfg(const GemmParams& p, hipStream_t s) {
    static bool attr_set = false;
    auto kern = conv_gemm_kernel<Cfg, KIND>;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                Cfg::kLdsBytes) != hipSuccess)
            return SPARQ_ELAUNCH;
        attr_set = true;
    }
    GemmParams q = p;
    q.tiles_m = (int)((p.M + Cfg::kTM - 1) / Cfg::kTM);
    q.tiles_n = (p.N + Cfg::kTN - 1) / Cfg::kTN;
    const int64_t blocks = (int64_t)q.tiles_m * q.tiles_n;
    if (blocks > 0x7FFFFFFF) return SPARQ_EUNSUPPORTED;
    kern<<<(unsigned)blocks, Cfg::kThreads, Cfg::kLdsBytes, s>>>(q);
    return launch_status();
}

template <class Cfg>
static sparq_status launch_kind(TrimKind kind, const GemmParams& p, hipStream_t s) {
    switch (kind) {
        case kTrimNone: return launch_cfg<Cfg, kTrimNone>(p, s);
        case kTrimFloor: return launch_cfg<Cfg, kTrimFloor>(p, s);
        case kTrimFloorPair: return launch_cfg<Cfg, kTrimFloorPair>(p, s);
        case kTrimFloorPairWide: return launch_cfg<Cfg, kTrimFloorPairWide>(p, s);
        case kTrimRound: return launch_cfg<Cfg, kTrimRound>(p, s);
        case kTrimRoundPair: return launch_cfg<Cfg, kTrimRoundPair>(p, s);
        default: return launch_cfg<Cfg, kTrimRoundPairWide>(p, s);
    }
}

}  // namespace sparq

using namespace sparq;

extern "C" size_t sparq_workspace_bytes(const sparq_conv_desc* desc, const sparq_mode* mode) {
    ConvGeom g;
    if (!conv_geom(desc, &g) || !mode_valid(mode)) return 0;
    if (g.Cp == g.C) return 0;
    return (size_t)round_up((int64_t)g.B * g.H * g.W * g.Cp, 256);
}

extern "C" sparq_status sparq_conv_gemm(const uint8_t* x, const void* packed_w, const sparq_conv_desc* desc,
                                        const sparq_mode* mode, int32_t* acc, const float* scale, float* out,
                                        void* workspace, size_t workspace_bytes, void* stream) {
    ConvGeom g;
    if (!x || !packed_w || !conv_geom(desc, &g) || !mode_valid(mode)) return SPARQ_EINVAL;
    if (!acc && !out) return SPARQ_EINVAL;
    if (out && !scale) return SPARQ_EINVAL;
    if (!aligned(x, 16) || !aligned(packed_w, 256) || (acc && !aligned(acc, 16)) || (out && !aligned(out, 16)) ||
        (scale && !aligned(scale, 16)))
        return SPARQ_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);

    const uint8_t* xin = x;
    TrimKind kind = trim_kind(mode);
    size_t x_bytes = g.x_bytes;
    if (g.Cp != g.C) {
        // Channel counts that are not a multiple of 16: trim into a channel-padded copy
        // first (pairs stay inside the row; padded channels are zeros with zero weights),
        // then contract the copy without further trimming.
        const size_t need = sparq_workspace_bytes(desc, mode);
        if (!workspace || !aligned(workspace, 256)) return SPARQ_EINVAL;
        if (workspace_bytes < need) return SPARQ_EWORKSPACE;
        x_bytes = (size_t)g.B * g.H * g.W * g.Cp;
        if (x_bytes >= kInvalidOffset) return SPARQ_EUNSUPPORTED;
        const sparq_status st = launch_trim_pad(x, static_cast<uint8_t*>(workspace), (int64_t)g.B * g.H * g.W, g.C,
                                                g.Cp, mode, s);
        if (st != SPARQ_OK) return st;
        xin = static_cast<const uint8_t*>(workspace);
        kind = kTrimNone;
    }
    if (x_bytes >= kInvalidOffset) return SPARQ_EUNSUPPORTED;

    GemmParams p{};
    p.x = xin;
    p.wpk = static_cast<const uint8_t*>(packed_w) + g.w_off;
    p.colsum = static_cast<const int32_t*>(packed_w);
    p.acc = acc;
    p.scale = scale;
    p.out = out;
    p.M = g.M;
    p.x_bytes = (uint32_t)x_bytes;
    p.N = g.N; p.Np = g.Np; p.Kk = g.Kk; p.nkb = g.Kp / kStepK;
    p.H = g.H; p.W = g.W; p.C = g.Cp; p.Ho = g.Ho; p.Wo = g.Wo; p.KH = g.KH; p.KW = g.KW;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw;
    p.luts = make_luts(mode->window_bits, mode->shift_mask);

    return launch_kind<TileCfg<128, 128, 2, 2>>(kind, p, s);
}
