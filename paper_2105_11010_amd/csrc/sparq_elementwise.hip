// Streaming kernels of libsparq: the standalone trim (Sections 3.1-3.2), the
// per-output-channel dequantisation (Section 5), the one-time weight packing
// and the trimmed, channel-padded copy used for channel counts that are not a
// multiple of 16.  All of them are bound by HBM traffic, so each lane moves
// 128-bit words and the grid is sized to a few workgroups per compute unit.
#include "sparq_common.h"

namespace sparq {

constexpr int kEwThreads = 256;
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef int v4s __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
// bytes read + written from which a streaming kernel takes the non-temporal form: the last-level cache holds 256 MiB
constexpr int64_t kStreamedBytes = (int64_t)256 << 20;

static int ew_grid(int64_t work_items, int per_block) {
    int64_t blocks = (work_items + per_block - 1) / per_block;
    const int64_t cap = 256 * 16;            // 256 compute units, 16 workgroups each
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

// ---- standalone trim ---------------------------------------------------------
// Even C: pairs (2j, 2j+1) of a row are also pairs of the flattened array, so
// the tensor is processed as one stream of 16-byte words.
// NT: non-temporal loads and stores, for tensors larger than the last-level cache that are streamed once (+8 % there;
// cache-resident or in-place tensors are faster with ordinary accesses).
template <int KIND, bool NT>
__global__ __launch_bounds__(kEwThreads) void trim_vec_kernel(const uint4* x, uint4* y,
                                                              int64_t n_vec, TrimLuts L) {
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < n_vec; i += stride) {
        const v4u* src = reinterpret_cast<const v4u*>(x) + i;
        v4u v = NT ? __builtin_nontemporal_load(src) : *src;
        v.x = trim4_kind<KIND>(v.x, L);
        v.y = trim4_kind<KIND>(v.y, L);
        v.z = trim4_kind<KIND>(v.z, L);
        v.w = trim4_kind<KIND>(v.w, L);
        if (NT) __builtin_nontemporal_store(v, reinterpret_cast<v4u*>(y) + i);
        else reinterpret_cast<v4u*>(y)[i] = v;
    }
}

// Any C, any alignment: one lane per pair of channels of one row.
template <int KIND>
__global__ __launch_bounds__(kEwThreads) void trim_pair_kernel(const uint8_t* x, uint8_t* y,
                                                               int64_t rows, int C, int64_t first_byte, TrimLuts L) {
    // first_byte > 0: C is even and only the flat tail [first_byte, rows*C) is handled here
    const int pairs = (C + 1) / 2;
    const int64_t total = first_byte > 0 ? (rows * C - first_byte) / 2 : rows * pairs;
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < total; i += stride) {
        int64_t off;
        bool has_b;
        if (first_byte > 0) {
            off = first_byte + 2 * i;
            has_b = true;
        } else {
            const int64_t r = i / pairs;
            const int c = (int)(i - r * pairs) * 2;
            off = r * C + c;
            has_b = c + 1 < C;
        }
        const uint32_t a = x[off];
        const uint32_t b = has_b ? x[off + 1] : 0u;
        const uint32_t t = trim4_kind<KIND>(a | (b << 8), L);
        y[off] = (uint8_t)t;
        if (has_b) y[off + 1] = (uint8_t)(t >> 8);
    }
}

template <int KIND>
static void launch_trim_kind(const uint8_t* x, uint8_t* y, int64_t rows, int C, const TrimLuts& L, hipStream_t s) {
    const int64_t bytes = rows * C;
    const bool vec_ok = (C % 2 == 0) && aligned(x, 16) && aligned(y, 16);
    int64_t done = 0;
    if (vec_ok && bytes >= 16) {
        const int64_t n_vec = bytes / 16;
        if (x != y && 2 * bytes >= kStreamedBytes)
            trim_vec_kernel<KIND, true><<<ew_grid(n_vec, kEwThreads * 4), kEwThreads, 0, s>>>(
                reinterpret_cast<const uint4*>(x), reinterpret_cast<uint4*>(y), n_vec, L);
        else
            trim_vec_kernel<KIND, false><<<ew_grid(n_vec, kEwThreads * 4), kEwThreads, 0, s>>>(
                reinterpret_cast<const uint4*>(x), reinterpret_cast<uint4*>(y), n_vec, L);
        done = n_vec * 16;
    }
    if (done < bytes) {
        const int64_t items = vec_ok ? (bytes - done) / 2 : rows * ((C + 1) / 2);
        trim_pair_kernel<KIND><<<ew_grid(items, kEwThreads), kEwThreads, 0, s>>>(x, y, rows, C, vec_ok ? done : 0, L);
    }
}

// ---- trimmed copy with channels padded to a multiple of 16 -------------------
template <int KIND>
__global__ __launch_bounds__(kEwThreads) void trim_pad_kernel(const uint8_t* __restrict__ x, uint32_t* __restrict__ xp,
                                                              int64_t pixels, int C, int Cp, TrimLuts L) {
    const int words = Cp / 4;
    const int64_t total = pixels * words;
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < total; i += stride) {
        const int64_t pix = i / words;
        const int c = (int)(i - pix * words) * 4;
        const uint8_t* src = x + pix * C + c;
        uint32_t v = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (c + j < C) v |= (uint32_t)src[j] << (8 * j);   // channels past C act as zeros (implicit zero partner)
        xp[i] = trim4_kind<KIND>(v, L);
    }
}

template <int KIND>
static void launch_trim_pad_kind(const uint8_t* x, uint8_t* xp, int64_t pixels, int C, int Cp, const TrimLuts& L,
                                 hipStream_t s) {
    const int64_t total = pixels * (Cp / 4);
    trim_pad_kernel<KIND><<<ew_grid(total, kEwThreads * 2), kEwThreads, 0, s>>>(x, reinterpret_cast<uint32_t*>(xp),
                                                                               pixels, C, Cp, L);
}

#define SPARQ_DISPATCH_KIND(kind, FN, ...)                                                  \
    switch (kind) {                                                                         \
        case kTrimNone: FN<kTrimNone>(__VA_ARGS__); break;                                  \
        case kTrimFloor: FN<kTrimFloor>(__VA_ARGS__); break;                                \
        case kTrimFloorPair: FN<kTrimFloorPair>(__VA_ARGS__); break;                        \
        case kTrimFloorPairWide: FN<kTrimFloorPairWide>(__VA_ARGS__); break;                \
        case kTrimRound: FN<kTrimRound>(__VA_ARGS__); break;                                \
        case kTrimRound4: FN<kTrimRound4>(__VA_ARGS__); break;                              \
        case kTrimRoundPair4: FN<kTrimRoundPair4>(__VA_ARGS__); break;                      \
        default: FN<kTrimRoundPairWide>(__VA_ARGS__); break;                                \
    }

sparq_status launch_trim_pad(const uint8_t* x, uint8_t* xp, int64_t pixels, int C, int Cp, const sparq_mode* mode,
                             hipStream_t stream) {
    const TrimLuts L = make_luts(mode->window_bits, mode->shift_mask);
    SPARQ_DISPATCH_KIND(trim_kind(mode), launch_trim_pad_kind, x, xp, pixels, C, Cp, L, stream);
    return launch_status();
}

// ---- dequantisation ----------------------------------------------------------
template <bool NT>
__global__ __launch_bounds__(kEwThreads) void dequant_vec_kernel(const int4* __restrict__ acc, const float* __restrict__ scale,
                                                                 float4* __restrict__ out, int64_t n_vec, int N) {
    // N % 4 == 0: a 16-byte word never straddles a row
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < n_vec; i += stride) {
        const int n = (int)((i * 4) % N);
        const v4s* src = reinterpret_cast<const v4s*>(acc) + i;
        const v4s a = NT ? __builtin_nontemporal_load(src) : *src;
        const float4 s = *reinterpret_cast<const float4*>(scale + n);
        v4f o;
        o.x = __fmul_rn((float)a.x, s.x);
        o.y = __fmul_rn((float)a.y, s.y);
        o.z = __fmul_rn((float)a.z, s.z);
        o.w = __fmul_rn((float)a.w, s.w);
        if (NT) __builtin_nontemporal_store(o, reinterpret_cast<v4f*>(out) + i);
        else reinterpret_cast<v4f*>(out)[i] = o;
    }
}

__global__ __launch_bounds__(kEwThreads) void dequant_scalar_kernel(const int32_t* __restrict__ acc, const float* __restrict__ scale,
                                                                    float* __restrict__ out, int64_t total, int N) {
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < total; i += stride)
        out[i] = __fmul_rn((float)acc[i], scale[i % N]);
}

// ---- requantisation to the next layer's unsigned 8-bit activations ------------
// y = clamp(round_to_nearest_even(acc * factor[n]), 0, 255), the product and the rounding in fp32
// (requant_u8 and the packing conversion instruction, which rounds and saturates the same way)
__global__ __launch_bounds__(kEwThreads) void requant_vec_kernel(const int4* __restrict__ acc, const float* __restrict__ factor,
                                                                 uint32_t* __restrict__ y, int64_t n_vec, int N) {
    // N % 4 == 0: a word of four results never straddles a row
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < n_vec; i += stride) {
        const int n = (int)((i * 4) % N);
        const int4 a = acc[i];
        const float4 f = *reinterpret_cast<const float4*>(factor + n);
        uint32_t w = __builtin_amdgcn_cvt_pk_u8_f32(__fmul_rn((float)a.x, f.x), 0, 0);
        w = __builtin_amdgcn_cvt_pk_u8_f32(__fmul_rn((float)a.y, f.y), 1, w);
        w = __builtin_amdgcn_cvt_pk_u8_f32(__fmul_rn((float)a.z, f.z), 2, w);
        y[i] = __builtin_amdgcn_cvt_pk_u8_f32(__fmul_rn((float)a.w, f.w), 3, w);
    }
}

__global__ __launch_bounds__(kEwThreads) void requant_scalar_kernel(const int32_t* __restrict__ acc, const float* __restrict__ factor,
                                                                    uint8_t* __restrict__ y, int64_t total, int N) {
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < total; i += stride)
        y[i] = (uint8_t)requant_u8(acc[i], factor[i % N]);
}

// ---- weight packing ----------------------------------------------------------
// packed[w_off + ((kb*4 + kc)*Np + n)*16 + j] = w[n][tap][c + j]  with  k = kb*64 + kc*16 = tap*Cp + c
__global__ __launch_bounds__(kEwThreads) void pack_weights_kernel(const int8_t* __restrict__ w, uint4* __restrict__ dst,
                                                                  int N, int Np, int C, int Cq, int taps, int Kp) {
    const int64_t total = (int64_t)(Kp / kChunk) * Np;
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < total; i += stride) {
        const int n = (int)(i % Np);
        const int k = (int)(i / Np) * kChunk;
        const int tap = k / Cq;
        const int c = k - tap * Cq;
        uint32_t v[4] = {0, 0, 0, 0};
        if (n < N && tap < taps) {
            const int8_t* src = w + ((int64_t)n * taps + tap) * C + c;
#pragma unroll
            for (int j = 0; j < kChunk; ++j)
                if (c + j < C) v[j >> 2] |= (uint32_t)(uint8_t)src[j] << (8 * (j & 3));
        }
        dst[i] = make_uint4(v[0], v[1], v[2], v[3]);
    }
}

// Weights of a pixel-folded layer (ConvGeom::fold): output channel n' = p * N + n of the folded
// problem holds, at tap (kh, kwf) and folded channel 4 * q + c, the weight w[n][kh][kw][c] of the
// original tap kw that super-pixel slot q lines up with for output class p (zero where there is none).
__global__ __launch_bounds__(kEwThreads) void pack_weights_fold_kernel(const int8_t* __restrict__ w, uint4* __restrict__ dst,
                                                                       int N, int Np, int C, int KH, int KW, int Kp,
                                                                       int P, int KWf, int kw_min, int sw, int pw) {
    const int64_t total = (int64_t)(Kp / kChunk) * Np;
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t i = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; i < total; i += stride) {
        const int nf = (int)(i % Np);
        const int tap = (int)(i / Np);              // one 16-byte chunk = one folded tap (kh, kwf)
        const int kh = tap / KWf, kwf = tap - kh * KWf;
        uint32_t v[4] = {0, 0, 0, 0};
        if (nf < P * N && kh < KH) {
            const int p = nf / N, n = nf - p * N;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int kw = 4 * (kwf + kw_min) + q - (sw * p - pw);
                if (kw < 0 || kw >= KW) continue;
                const int8_t* src = w + (((int64_t)n * KH + kh) * KW + kw) * C;
                for (int c = 0; c < C; ++c) v[q] |= (uint32_t)(uint8_t)src[c] << (8 * c);
            }
        }
        dst[i] = make_uint4(v[0], v[1], v[2], v[3]);
    }
}

// colsum[n] = sum_k w[n % N][k]; one wavefront per (possibly replicated) output channel
__global__ __launch_bounds__(64) void weight_colsum_kernel(const int8_t* __restrict__ w, int32_t* __restrict__ colsum, int N,
                                                           int Nrep, int K) {
    const int n = (int)blockIdx.x < Nrep ? (int)blockIdx.x % N : N;
    int32_t s = 0;
    if (n < N)
        for (int k = threadIdx.x; k < K; k += 64) s += w[(int64_t)n * K + k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
    if (threadIdx.x == 0) colsum[blockIdx.x] = s;
}

}  // namespace sparq

using namespace sparq;

extern "C" sparq_status sparq_trim(const uint8_t* x, uint8_t* y, int64_t rows, int32_t C, const sparq_mode* mode,
                                   void* stream) {
    if (rows < 0 || C <= 0 || !mode_valid(mode)) return SPARQ_EINVAL;
    if (rows == 0) return SPARQ_OK;          // empty input: nothing to read or write
    if (!x || !y) return SPARQ_EINVAL;
    if (rows > (INT64_MAX / 4) / C) return SPARQ_EINVAL;
    const int64_t bytes = rows * C;
    if (x != y) {
        const uintptr_t xa = (uintptr_t)x, ya = (uintptr_t)y;
        if (xa < ya + (uint64_t)bytes && ya < xa + (uint64_t)bytes) return SPARQ_EINVAL;   // partial overlap
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const TrimKind kind = trim_kind(mode);
    if (kind == kTrimNone) {
        if (x != y && hipMemcpyAsync(y, x, (size_t)bytes, hipMemcpyDeviceToDevice, s) != hipSuccess) return SPARQ_ELAUNCH;
        return SPARQ_OK;
    }
    const TrimLuts L = make_luts(mode->window_bits, mode->shift_mask);
    SPARQ_DISPATCH_KIND(kind, launch_trim_kind, x, y, rows, C, L, s);
    return launch_status();
}

extern "C" sparq_status sparq_dequant(const int32_t* acc, const float* scale, float* out, int64_t M, int32_t N,
                                      void* stream) {
    if (M < 0 || N <= 0) return SPARQ_EINVAL;
    if (M == 0) return SPARQ_OK;
    if (!acc || !scale || !out) return SPARQ_EINVAL;
    if (M > (INT64_MAX / 8) / N) return SPARQ_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t total = M * N;
    if (N % 4 == 0 && aligned(acc, 16) && aligned(out, 16) && aligned(scale, 16)) {
        const int64_t n_vec = total / 4;
        if (8 * total >= kStreamedBytes)
            dequant_vec_kernel<true><<<ew_grid(n_vec, kEwThreads * 4), kEwThreads, 0, s>>>(
                reinterpret_cast<const int4*>(acc), scale, reinterpret_cast<float4*>(out), n_vec, N);
        else
            dequant_vec_kernel<false><<<ew_grid(n_vec, kEwThreads * 4), kEwThreads, 0, s>>>(
                reinterpret_cast<const int4*>(acc), scale, reinterpret_cast<float4*>(out), n_vec, N);
    } else {
        dequant_scalar_kernel<<<ew_grid(total, kEwThreads * 4), kEwThreads, 0, s>>>(acc, scale, out, total, N);
    }
    return launch_status();
}

extern "C" sparq_status sparq_requant(const int32_t* acc, const float* factor, uint8_t* y, int64_t M, int32_t N,
                                      void* stream) {
    if (M < 0 || N <= 0) return SPARQ_EINVAL;
    if (M == 0) return SPARQ_OK;
    if (!acc || !factor || !y) return SPARQ_EINVAL;
    if (M > (INT64_MAX / 8) / N) return SPARQ_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t total = M * N;
    if (N % 4 == 0 && aligned(acc, 16) && aligned(y, 4) && aligned(factor, 16)) {
        const int64_t n_vec = total / 4;
        requant_vec_kernel<<<ew_grid(n_vec, kEwThreads * 4), kEwThreads, 0, s>>>(
            reinterpret_cast<const int4*>(acc), factor, reinterpret_cast<uint32_t*>(y), n_vec, N);
    } else {
        requant_scalar_kernel<<<ew_grid(total, kEwThreads * 4), kEwThreads, 0, s>>>(acc, factor, y, total, N);
    }
    return launch_status();
}

extern "C" size_t sparq_packed_bytes(const sparq_conv_desc* desc) {
    ConvGeom g;
    return conv_geom(desc, &g) ? g.packed_bytes : 0;
}

extern "C" sparq_status sparq_pack_weights(const int8_t* w, const sparq_conv_desc* desc, void* packed,
                                           size_t packed_bytes, void* stream) {
    ConvGeom g;
    if (!w || !packed || !conv_geom(desc, &g) || !aligned(packed, 256)) return SPARQ_EINVAL;
    if (packed_bytes < g.packed_bytes) return SPARQ_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* base = static_cast<uint8_t*>(packed);
    weight_colsum_kernel<<<g.Np, 64, 0, s>>>(w, reinterpret_cast<int32_t*>(base), g.N, g.fold_p * g.N, g.K);
    const int64_t chunks = (int64_t)(g.Kp / kChunk) * g.Np;
    if (g.fold)
        pack_weights_fold_kernel<<<ew_grid(chunks, kEwThreads), kEwThreads, 0, s>>>(
            w, reinterpret_cast<uint4*>(base + g.w_off), g.N, g.Np, g.C, g.KH, g.KW, g.Kp, g.fold_p, g.fold_kw,
            g.fold_kw_min, g.sw, g.pw);
    else
        pack_weights_kernel<<<ew_grid(chunks, kEwThreads), kEwThreads, 0, s>>>(
            w, reinterpret_cast<uint4*>(base + g.w_off), g.N, g.Np, g.C, g.Cq, g.KH * g.KW, g.Kp);
    return launch_status();
}

extern "C" const char* sparq_strerror(sparq_status status) {
    switch (status) {
        case SPARQ_OK: return "ok";
        case SPARQ_EINVAL: return "invalid argument";
        case SPARQ_EUNSUPPORTED: return "unsupported configuration";
        case SPARQ_EWORKSPACE: return "buffer too small";
        case SPARQ_ELAUNCH: return "HIP launch failed";
        default: return "unknown status";
    }
}
